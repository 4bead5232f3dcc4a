// Device-side helpers shared by the libpe kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pe {

// Storage type of a bfloat16 element (the kernels only ever move or widen it).
struct bf16_t {
  uint16_t bits;
};

constexpr int kWave = 64;

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int kPerVec = 4;  // elements in one 16-byte lane load
};
template <>
struct Elem<bf16_t> {
  static constexpr int kPerVec = 8;
};

// Geometry of a [tokens][D] page when every lane loads 16 bytes and consecutive lanes load
// consecutive addresses: kLanesPerRow lanes cover one token row, one wave-load covers
// kTokensPerLoad token rows.
template <typename T, int D>
struct RowGeom {
  static constexpr int kPerVec = Elem<T>::kPerVec;
  static constexpr int kLanesPerRow = D / kPerVec;
  static constexpr int kTokensPerLoad = kWave / kLanesPerRow;
  static_assert(kLanesPerRow >= 8 && kLanesPerRow <= 32, "unsupported head_dim / dtype");
};

__device__ __forceinline__ float bf16_lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (inputs are finite or inf; NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Widen element e (0 .. kPerVec-1) of a 16-byte vector to fp32.
template <typename T>
__device__ __forceinline__ float vec_elem(const uint4& v, int e);
template <>
__device__ __forceinline__ float vec_elem<float>(const uint4& v, int e) {
  const uint32_t w = e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
  return __uint_as_float(w);
}
template <>
__device__ __forceinline__ float vec_elem<bf16_t>(const uint4& v, int e) {
  const int i = e >> 1;
  const uint32_t w = i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
  return (e & 1) ? bf16_hi_to_f32(w) : bf16_lo_to_f32(w);
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// Value of `v` in lane (lane ^ M).  M = 1, 2: DPP quad permute; 4, 8, 16: ds_swizzle in bit-mask
// mode (works inside each half-wave); 32: ds_bpermute.
template <int M>
__device__ __forceinline__ int lane_xor_i32(int v) {
  static_assert(M == 1 || M == 2 || M == 4 || M == 8 || M == 16 || M == 32, "power of two < 64");
  if constexpr (M == 1) {
    return __builtin_amdgcn_update_dpp(0, v, 0xB1 /* quad_perm [1,0,3,2] */, 0xf, 0xf, true);
  } else if constexpr (M == 2) {
    return __builtin_amdgcn_update_dpp(0, v, 0x4E /* quad_perm [2,3,0,1] */, 0xf, 0xf, true);
  } else if constexpr (M == 32) {
    return __builtin_amdgcn_ds_bpermute((lane_id() ^ 32) << 2, v);
  } else {
    return __builtin_amdgcn_ds_swizzle(v, (M << 10) | 0x1f);
  }
}
template <int M>
__device__ __forceinline__ float lane_xor_f32(float v) {
  return __int_as_float(lane_xor_i32<M>(__float_as_int(v)));
}
template <int M>
__device__ __forceinline__ double lane_xor_f64(double v) {
  const int lo = lane_xor_i32<M>(__double2loint(v));
  const int hi = lane_xor_i32<M>(__double2hiint(v));
  return __hiloint2double(hi, lo);
}

// Value of lane ((lane & ~(W-1)) | J): broadcast of position J of every aligned group of W lanes.
template <int W, int J>
__device__ __forceinline__ float group_bcast_f32(float v) {
  static_assert(W == 1 || W == 2 || W == 4 || W == 8, "group width");
  static_assert(J >= 0 && J < W, "position inside the group");
  if constexpr (W == 1) {
    return v;
  } else if constexpr (W == 2) {  // quad positions 0,1 read position J; positions 2,3 read position 2+J
    constexpr int ctrl = J | (J << 2) | ((2 | J) << 4) | ((2 | J) << 6);
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, 0xf, 0xf, true));
  } else if constexpr (W == 4) {  // quad_perm [J,J,J,J]
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), J * 0x55, 0xf, 0xf, true));
  } else {
    // ds_swizzle bit-mask mode: lane' = ((lane & and) | or) ^ xor inside each half-wave
    return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), (J << 5) | 0x18));
  }
}

template <int BITS>
__host__ __device__ constexpr int bit_reverse(int x) {
  int r = 0;
  for (int i = 0; i < BITS; ++i) r |= ((x >> i) & 1) << (BITS - 1 - i);
  return r;
}

__host__ __device__ constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x >> 1); }

// 16-byte global load of lane-consecutive data.
__device__ __forceinline__ uint4 load_vec(const void* base, int64_t vec_index) {
  return reinterpret_cast<const uint4*>(base)[vec_index];
}

// The same load with a non-temporal hint: K/V pages are read once per launch and should not displace
// tables, queries and partials from the caches.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_vec_stream(const void* base, int64_t vec_index) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(base) + vec_index);
  return make_uint4(v.x, v.y, v.z, v.w);
}

}  // namespace pe
