// Device-side helpers: bf16 storage conversion, 16-byte vector loads, wavefront
// and workgroup reductions.  gfx950 only (64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mdi_internal.h"

namespace mdi {

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even, the rounding the input recipe uses for stored tensors
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> struct Storage;
template <> struct Storage<float> {
  static constexpr int kVec = 4;  // elements per 16-byte load
  __device__ static __forceinline__ void load(const float* p, float (&v)[4]) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  __device__ static __forceinline__ float get(const float* p) { return *p; }
  __device__ static __forceinline__ void put(float* p, float v) { *p = v; }
};
template <> struct Storage<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    const uint4 t = *reinterpret_cast<const uint4*>(p);
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
    v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xFFFF0000u);
    v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xFFFF0000u);
  }
  __device__ static __forceinline__ float get(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static __forceinline__ void put(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

__device__ __forceinline__ float load_kind(const void* p, int kind, long i) {
  return kind == IN_BF16 ? bf16_to_f32(((const bf16_t*)p)[i]) : ((const float*)p)[i];
}
__device__ __forceinline__ void store_kind(void* p, int kind, long i, float v) {
  if (kind == IN_BF16) ((bf16_t*)p)[i] = f32_to_bf16(v); else ((float*)p)[i] = v;
}

// Cross-lane adds through the DPP data path (full VALU rate, no LDS crossbar round trip).
// Lanes a control word does not write receive 0 and so add nothing.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false);
  return v + __int_as_float(moved);
}
constexpr int kDppXor1 = 0xB1;          // quad_perm:[1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm:[2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // lane i <-> 7 - i inside groups of 8
constexpr int kDppMirror = 0x140;       // lane i <-> 15 - i inside rows of 16
constexpr int kDppBcast15 = 0x142;      // lane 15 of each row -> every lane of the next row
constexpr int kDppBcast31 = 0x143;      // lane 31 -> every lane of rows 2 and 3

// Sum over the 64 lanes; the total is valid in lane 63 only.
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
  v = dpp_add<kDppXor1, 0xF>(v);
  v = dpp_add<kDppXor2, 0xF>(v);
  v = dpp_add<kDppHalfMirror, 0xF>(v);
  v = dpp_add<kDppMirror, 0xF>(v);       // every lane of a row holds the row's sum
  v = dpp_add<kDppBcast15, 0xA>(v);      // rows 1 and 3 add the sum of rows 0 and 2
  v = dpp_add<kDppBcast31, 0xC>(v);      // rows 2 and 3 add lane 31 = rows 0 + 1
  return v;
}

// Sum inside aligned groups of L lanes (L a power of two), result in every lane of the group.
__device__ __forceinline__ float group_sum(float v, int L) {
  if (L >= 2) v = dpp_add<kDppXor1, 0xF>(v);
  if (L >= 4) v = dpp_add<kDppXor2, 0xF>(v);
  if (L >= 8) v = dpp_add<kDppHalfMirror, 0xF>(v);
  if (L >= 16) v = dpp_add<kDppMirror, 0xF>(v);
  if (L >= 32) v += __shfl_xor(v, 16, 64);
  if (L >= 64) v += __shfl_xor(v, 32, 64);
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Sum over the workgroup; every thread gets the result.  `red` holds >= 4 floats
// of LDS that the caller does not otherwise touch during the call.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += red[w];
  return t;
}

__device__ __forceinline__ float gelu_tanh_f(float x) {
  const float k = 0.7978845608028654f;  // sqrt(2/pi)
  return 0.5f * x * (1.f + tanhf(k * (x + 0.044715f * x * x * x)));
}
__device__ __forceinline__ float gelu_erf_f(float x) { return 0.5f * x * (1.f + erff(x * 0.7071067811865476f)); }
__device__ __forceinline__ float silu_f(float x) { return x / (1.f + __expf(-x)); }


// A token id read from device memory indexes the embedding table, so it is checked where it is read: an id outside
// [0, vocab) raises the partition's error word (value 2) and is replaced by token 0.
__device__ __forceinline__ long checked_token(const void* in, long index, int vocab, int* err) {
  const long tok = ((const int32_t*)in)[index];
  if (tok < 0 || tok >= vocab) {
    if (err) __hip_atomic_store(err, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return 0;
  }
  return tok;
}

}  // namespace mdi
