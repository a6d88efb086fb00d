// Shared device helpers for the libquoka kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "quoka.h"

namespace quoka {

constexpr float kNormEps = 1e-8f;  // lower clamp of every vector norm
constexpr int kWave = 64;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Kernel-side view of quoka_shape (plain copy; passed by value).
struct Dims {
  int b, n_q, n_kv, g, d, C, T_max, n_ret, B_max;
  int flags;   // QUOKA_SCORE_* bits
  long long qs[3], kvs[3], cks[3], os[3];
};

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// Round-to-nearest-even fp32 -> bf16 bit pattern (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Order-preserving map float -> uint32: a < b  <=>  okey(a) < okey(b).
__device__ __forceinline__ uint32_t okey(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Element loads widened to float.  T = float or uint16_t (bf16 bits).
template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int kPer16B = 4;
  __device__ static __forceinline__ void load8(const float* p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  __device__ static __forceinline__ float load1(const float* p) { return *p; }
};
template <>
struct Elem<uint16_t> {
  static constexpr int kPer16B = 8;
  __device__ static __forceinline__ void load8(const uint16_t* p, float (&v)[8]) {
    const uint4 a = *reinterpret_cast<const uint4*>(p);
    v[0] = __uint_as_float(a.x << 16); v[1] = __uint_as_float(a.x & 0xFFFF0000u);
    v[2] = __uint_as_float(a.y << 16); v[3] = __uint_as_float(a.y & 0xFFFF0000u);
    v[4] = __uint_as_float(a.z << 16); v[5] = __uint_as_float(a.z & 0xFFFF0000u);
    v[6] = __uint_as_float(a.w << 16); v[7] = __uint_as_float(a.w & 0xFFFF0000u);
  }
  __device__ static __forceinline__ float load1(const uint16_t* p) { return bf16_bits_to_f32(*p); }
};

// Sum over the lanes of an aligned group of W lanes (W power of two <= 64); every lane gets the sum.
template <int W>
__device__ __forceinline__ float group_sum(float x) {
#pragma unroll
  for (int o = W / 2; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}
template <int W>
__device__ __forceinline__ float group_max(float x) {
#pragma unroll
  for (int o = W / 2; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, kWave));
  return x;
}

// Sum over each aligned group of 16 lanes (one DPP row) with four row rotations: plain VALU work, no LDS
// crossbar traffic.  Every lane of the group gets the sum.
__device__ __forceinline__ float row16_sum(float x) {
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x128, 0xF, 0xF, false));   // row_ror:8
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x124, 0xF, 0xF, false));   // row_ror:4
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x122, 0xF, 0xF, false));   // row_ror:2
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x121, 0xF, 0xF, false));   // row_ror:1
  return x;
}

// Sum over the 64 lanes of a wave: DPP inside each 16-lane row, then two cross-row exchanges.
__device__ __forceinline__ float wave64_sum(float x) {
  x = row16_sum(x);
  x += __shfl_xor(x, 16, kWave);
  x += __shfl_xor(x, 32, kWave);
  return x;
}

// Exchange between lane l and lane l^32 through v_permlane32_swap: returns the partner's value.
__device__ __forceinline__ float other_half(float x) {
  const uint32_t u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // r[0] = {x[0..31], x[0..31]}, r[1] = {x[32..63], x[32..63]}
  const uint32_t lo = r[0], hi = r[1];
  return __uint_as_float((threadIdx.x & 32) ? lo : hi);
}

// Exclusive prefix sum of one uint per thread over a block of NT threads (NT multiple of 64, <= 1024).
// `wsum` is LDS scratch of at least NT/64 + 1 uints.  Returns the exclusive prefix; *total gets the block sum.
template <int NT>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t x, uint32_t* wsum, uint32_t* total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t inc = x;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(inc, o, kWave);
    if (lane >= o) inc += y;
  }
  __syncthreads();  // protect wsum against a previous use
  if (lane == 63) wsum[w] = inc;
  __syncthreads();
  if (w == 0) {   // wave 0 scans the NT/64 wave totals
    const uint32_t t = lane < NT / 64 ? wsum[lane] : 0u;
    uint32_t run = t;
#pragma unroll
    for (int o = 1; o < NT / 64; o <<= 1) {
      const uint32_t y = __shfl_up(run, o, kWave);
      if (lane >= o) run += y;
    }
    if (lane < NT / 64) wsum[lane] = run - t;
    if (lane == NT / 64 - 1) wsum[NT / 64] = run;
  }
  __syncthreads();
  *total = wsum[NT / 64];
  return wsum[w] + inc - x;
}

// One wave (the caller guarantees threadIdx.x < 64 and all 64 lanes active) walks a 256-bin LDS
// histogram in descending (DESC) or ascending bin order and finds the bin in which the running count
// reaches `need` (1-based rank, need <= total count).  The one lane that finds it ORs the bin, shifted,
// into *prefix_io and stores the rank remaining inside the bin to *need_out.
template <bool DESC>
__device__ __forceinline__ void wave_find_bin256(const uint32_t* hist, uint32_t need, int shift, uint32_t* prefix_io,
                                                 uint32_t* need_out) {
  const int lane = threadIdx.x & 63;
  uint32_t c[4];
  uint32_t sum = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int o = 4 * lane + j;   // position in scan order
    c[j] = hist[DESC ? 255 - o : o];
    sum += c[j];
  }
  uint32_t inc = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(inc, o, kWave);
    if (lane >= o) inc += y;
  }
  const uint32_t excl = inc - sum;
  if (excl < need && need <= inc) {   // exactly one lane
    uint32_t rem = need - excl;
    int j = 0;
#pragma unroll
    for (; j < 3; ++j) {
      if (rem <= c[j]) break;
      rem -= c[j];
    }
    const int o = 4 * lane + j;
    *prefix_io |= (uint32_t)(DESC ? 255 - o : o) << shift;
    *need_out = rem;
  }
}

}  // namespace quoka
