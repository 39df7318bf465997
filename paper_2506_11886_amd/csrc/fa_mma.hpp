// Matrix-core fragments for gfx950, 64-lane wavefronts.
//
// One logical step contracts 32 values of k into a 16x16 fp32 tile:
//   acc[i][j] += sum_k A[i][k] * B[k][j]
// Register layout (identical for every element type):
//   A fragment: lane l holds row  i = l % 16, the 8 k-values of slot group l / 16
//   B fragment: lane l holds col  j = l % 16, the 8 k-values of slot group l / 16
//   acc       : lane l holds col  j = l % 16, rows i = 4 * (l / 16) + {0,1,2,3}
// The hardware multiplies A's (group, element) with B's (group, element), so
// which 8 k-values a group holds is the caller's choice as long as A and B
// agree.  16-bit types take one v_mfma_f32_16x16x32; fp32 takes eight
// v_mfma_f32_16x16x4_f32, one per element of the group.
#pragma once

#include <hip/hip_runtime.h>

#include "fa_common.hpp"

namespace fa {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct f16_t { uint16_t bits; };

template <typename T> struct Frag;

template <> struct Frag<bf16_t> {
  u32x4 v;  // 8 bf16
  __device__ __forceinline__ void zero() { v = u32x4{0u, 0u, 0u, 0u}; }
  // 16-byte aligned source of 8 consecutive elements
  __device__ __forceinline__ void load(const bf16_t* p) { v = *reinterpret_cast<const u32x4*>(p); }
  __device__ __forceinline__ void set(int e, float x) {
    const uint32_t b = f32_to_bf16(x);
    uint32_t w = v[e >> 1];
    w = (e & 1) ? ((w & 0x0000ffffu) | (b << 16)) : ((w & 0xffff0000u) | b);
    v[e >> 1] = w;
  }
};

template <> struct Frag<f16_t> {
  u32x4 v;  // 8 fp16
  __device__ __forceinline__ void zero() { v = u32x4{0u, 0u, 0u, 0u}; }
  __device__ __forceinline__ void load(const f16_t* p) { v = *reinterpret_cast<const u32x4*>(p); }
};

template <> struct Frag<float> {
  float v[8];
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = 0.0f;
  }
  __device__ __forceinline__ void load(const float* p) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(p);
    const f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
    v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
    v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
  }
  __device__ __forceinline__ void set(int e, float x) { v[e] = x; }
};

__device__ __forceinline__ void mma_k32(f32x4& acc, const Frag<bf16_t>& a, const Frag<bf16_t>& b) {
  acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a.v),
                                                __builtin_bit_cast(bf16x8, b.v), acc, 0, 0, 0);
}
__device__ __forceinline__ void mma_k32(f32x4& acc, const Frag<f16_t>& a, const Frag<f16_t>& b) {
  acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a.v),
                                               __builtin_bit_cast(f16x8, b.v), acc, 0, 0, 0);
}
__device__ __forceinline__ void mma_k32(f32x4& acc, const Frag<float>& a, const Frag<float>& b) {
#pragma unroll
  for (int e = 0; e < 8; ++e)
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[e], b.v[e], acc, 0, 0, 0);
}

}  // namespace fa
