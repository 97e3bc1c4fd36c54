// Device-side helpers shared by the kernels: wavefront reductions and masked float4 access.
#pragma once

#include "lopt_internal.h"

namespace lopt {

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over the 64 lanes of a wavefront; every lane gets the result. Fixed order.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_f<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_f<0x141>(v);  // row_half_mirror
  v += dpp_f<0x140>(v);  // row_mirror: every lane of a row of 16 holds the row's sum
  float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
  float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
  float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
  float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
  return (a + b) + (c + d);
}

typedef float f32x4n __attribute__((ext_vector_type(4)));

// Load four consecutive floats starting at column `col` of a row of length n whose first
// element is at `row`. VEC: the address is 16-byte aligned and n % 4 == 0.
template <bool VEC>
__device__ __forceinline__ float4 load4(const float* __restrict__ row, int col, int n) {
  if (VEC) {
    if (col < n) return *reinterpret_cast<const float4*>(row + col);
    return make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (col < n) v.x = row[col];
  if (col + 1 < n) v.y = row[col + 1];
  if (col + 2 < n) v.z = row[col + 2];
  if (col + 3 < n) v.w = row[col + 3];
  return v;
}

template <bool VEC>
__device__ __forceinline__ void store4(float* __restrict__ row, int col, int n, float4 v) {
  if (VEC) {
    if (col < n) *reinterpret_cast<float4*>(row + col) = v;
    return;
  }
  if (col < n) row[col] = v.x;
  if (col + 1 < n) row[col + 1] = v.y;
  if (col + 2 < n) row[col + 2] = v.z;
  if (col + 3 < n) row[col + 3] = v.w;
}

// The same for the big streamed arrays (g, p, M, V): every element is touched once per pass and the
// working set is far larger than the caches, so the accesses are marked nontemporal (measured +5 % on a
// 6-read/4-write stream).
template <bool VEC>
__device__ __forceinline__ float4 load4s(const float* __restrict__ row, int col, int n) {
  if (VEC) {
    if (col < n) {
      const f32x4n v = __builtin_nontemporal_load(reinterpret_cast<const f32x4n*>(row + col));
      return make_float4(v.x, v.y, v.z, v.w);
    }
    return make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (col < n) v.x = __builtin_nontemporal_load(row + col);
  if (col + 1 < n) v.y = __builtin_nontemporal_load(row + col + 1);
  if (col + 2 < n) v.z = __builtin_nontemporal_load(row + col + 2);
  if (col + 3 < n) v.w = __builtin_nontemporal_load(row + col + 3);
  return v;
}

template <bool VEC>
__device__ __forceinline__ void store4s(float* __restrict__ row, int col, int n, float4 v) {
  if (VEC) {
    if (col < n) {
      const f32x4n w = {v.x, v.y, v.z, v.w};
      __builtin_nontemporal_store(w, reinterpret_cast<f32x4n*>(row + col));
    }
    return;
  }
  if (col < n) __builtin_nontemporal_store(v.x, row + col);
  if (col + 1 < n) __builtin_nontemporal_store(v.y, row + col + 1);
  if (col + 2 < n) __builtin_nontemporal_store(v.z, row + col + 2);
  if (col + 3 < n) __builtin_nontemporal_store(v.w, row + col + 3);
}

__device__ __forceinline__ float get(const float4& v, int i) {
  return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
}


}  // namespace lopt
