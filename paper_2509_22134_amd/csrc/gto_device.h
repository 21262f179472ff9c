// Device-side helpers shared by the GTO kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gto {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr float kLog2e = 1.44269504088896340736f;   // fp32(log2 e)
constexpr double kLn2 = 0.693147180559945309417232121458;
constexpr int kNoId = 0x7fffffff;                   // id of an empty top-k entry (loses every tie)

__device__ __forceinline__ float neg_inf() { return -__builtin_inff(); }

__device__ __forceinline__ int lane_id() {
  return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// lane i receives the value of lane i-1; lane 0 receives `fill`.
__device__ __forceinline__ int wave_shr1(int v, int fill) {
  return __builtin_amdgcn_update_dpp(fill, v, 0x138 /* wave_shr:1 */, 0xf, 0xf, false);
}
__device__ __forceinline__ float wave_shr1(float v, float fill) {
  return __int_as_float(wave_shr1(__float_as_int(v), __float_as_int(fill)));
}

__device__ __forceinline__ float readlane(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ int readlane(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}
__device__ __forceinline__ int wave_min(int v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = min(v, __shfl_xor(v, off, kWave));
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// (value, id) ordering used everywhere: larger value first, lower id first among equals.
__device__ __forceinline__ bool better(float v, int id, float w, int jd) {
  return (v > w) || (v == w && id < jd);
}

// Monotone map of an fp32 score to uint32 (larger float -> larger uint); -0 and +0 coincide.
__device__ __forceinline__ uint32_t ordered_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// 16 bytes of logits -> fp32 values.
template <typename T> struct Elem;
template <> struct Elem<uint16_t> {           // bf16 storage
  static constexpr int kPerVec = 8;
  __device__ static __forceinline__ void unpack(const u32x4 &q, float *x) {
    x[0] = __uint_as_float(q.x << 16); x[1] = __uint_as_float(q.x & 0xffff0000u);
    x[2] = __uint_as_float(q.y << 16); x[3] = __uint_as_float(q.y & 0xffff0000u);
    x[4] = __uint_as_float(q.z << 16); x[5] = __uint_as_float(q.z & 0xffff0000u);
    x[6] = __uint_as_float(q.w << 16); x[7] = __uint_as_float(q.w & 0xffff0000u);
  }
  __device__ static __forceinline__ float load1(const uint16_t *p) {
    return __uint_as_float(((uint32_t)*p) << 16);
  }
};
template <> struct Elem<float> {
  static constexpr int kPerVec = 4;
  __device__ static __forceinline__ void unpack(const u32x4 &q, float *x) {
    x[0] = __uint_as_float(q.x); x[1] = __uint_as_float(q.y);
    x[2] = __uint_as_float(q.z); x[3] = __uint_as_float(q.w);
  }
  __device__ static __forceinline__ float load1(const float *p) { return *p; }
};

// Offset (in elements) of slot (l, j) of root r, and the index of its statistics entry.
__device__ __forceinline__ int64_t stat_index(int r, int l, int j, int d, int k) {
  return ((int64_t)r * d + l) * k + j;
}

}  // namespace gto
