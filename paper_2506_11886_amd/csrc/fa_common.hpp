// Shared device/host helpers for the gfx950 FourierAttention kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "fourier_attn.h"

namespace fa {

// Per-kernel timing of the *_timed entry points: every launch carries its own start / stop
// event pair, which the runtime stamps with the dispatch's begin and end on the GPU (the
// interval between two ordinary stream events would also hold the launch latency).
struct KernelTimers {
  static constexpr int kMax = 3;
  hipEvent_t start[kMax] = {nullptr, nullptr, nullptr};
  hipEvent_t stop[kMax] = {nullptr, nullptr, nullptr};
  bool used[kMax] = {false, false, false};
  int create() {
    for (int i = 0; i < kMax; ++i)
      if (hipEventCreate(&start[i]) != hipSuccess || hipEventCreate(&stop[i]) != hipSuccess) return FA_ERR_HIP;
    return FA_OK;
  }
  void destroy() {
    for (int i = 0; i < kMax; ++i) {
      if (start[i]) (void)hipEventDestroy(start[i]);
      if (stop[i]) (void)hipEventDestroy(stop[i]);
    }
  }
  // milliseconds of kernels 0 .. n-1 (0 for a kernel that was not launched); waits for the last one
  int read(int n, float* ms) {
    for (int i = 0; i < n; ++i) {
      ms[i] = 0.0f;
      if (!used[i]) continue;
      if (hipEventSynchronize(stop[i]) != hipSuccess) return FA_ERR_HIP;
      if (hipEventElapsedTime(&ms[i], start[i], stop[i]) != hipSuccess) return FA_ERR_HIP;
    }
    return FA_OK;
  }
};
// launch, with the timers' event pair number i_ when timers are given (the plain launch is kept
// for the untimed entry points, which callers may record into a HIP graph)
#define FA_LAUNCH_TIMED(tm_, i_, kern_, grid_, block_, lds_, st_, ...)                               \
  do {                                                                                              \
    if (tm_) {                                                                                      \
      hipExtLaunchKernelGGL(kern_, grid_, block_, lds_, st_, (tm_)->start[i_], (tm_)->stop[i_], 0,  \
                            __VA_ARGS__);                                                           \
      (tm_)->used[i_] = true;                                                                       \
    } else {                                                                                        \
      hipLaunchKernelGGL(kern_, grid_, block_, lds_, st_, __VA_ARGS__);                             \
    }                                                                                               \
  } while (0)

constexpr int kWave = 64;

// ---------------------------------------------------------------------------
// element types
// ---------------------------------------------------------------------------
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
// round-to-nearest-even; NaN kept quiet
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kDtype = FA_F32;
  __device__ static __forceinline__ float load(const float* p) { return *p; }
  __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kDtype = FA_BF16;
  __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(p->bits); }
  __device__ static __forceinline__ void store(bf16_t* p, float v) { p->bits = f32_to_bf16(v); }
};

// ---------------------------------------------------------------------------
// basis: phi_m at integer position pos for period T (Eq. 4, zero row dropped)
// ---------------------------------------------------------------------------
// cos and sin of 2*pi*((n*pos) mod T)/T with the phase reduced in exact
// integer arithmetic, so that n*pos beyond 2^24 loses nothing.
__device__ __forceinline__ void unit_phase(int n, int pos, int T, float* c, float* s) {
  const uint32_t r = static_cast<uint32_t>((static_cast<uint64_t>(n) * static_cast<uint64_t>(pos)) %
                                           static_cast<uint64_t>(T));
  // sincospi takes half-turns: angle = pi * (2 r / T), 2r/T in [0, 2)
  const float x = 2.0f * (static_cast<float>(r) / static_cast<float>(T));
  sincospif(x, s, c);
}

// inverse squared norm over one period of the basis function of order n
__host__ __device__ __forceinline__ float basis_weight(int n, int T) {
  return (n == 0 || 2 * n == T) ? 1.0f / static_cast<float>(T) : 2.0f / static_cast<float>(T);
}

// ---------------------------------------------------------------------------
// wave / block reductions
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace fa
