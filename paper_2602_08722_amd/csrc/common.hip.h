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
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

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

// Sum over each aligned group of 16 lanes (one DPP row) with four row rotations: plain VALU work, no LDS
// crossbar traffic.  Every lane of the group gets the sum.
__device__ __forceinline__ float row16_sum(float x) {
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x128, 0xF, 0xF, false));   // row_ror:8
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x124, 0xF, 0xF, false));   // row_ror:4
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x122, 0xF, 0xF, false));   // row_ror:2
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x121, 0xF, 0xF, false));   // row_ror:1
  return x;
}

// Cross-lane steps on the VALU's DPP path (no LDS crossbar, a few clocks each instead of a ds_bpermute round trip).
// CTRL: row_shr:n = 0x110 + n (lane i reads lane i-n of its 16-lane row), row_bcast:15 = 0x142 (lane 15 of every row to
// the next row), row_bcast:31 = 0x143 (lane 31 to rows 2 and 3).  A lane without a source, or in a row that ROW_MASK
// leaves out, gets `idle`.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp_take(uint32_t idle, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)idle, (int)v, CTRL, ROW_MASK, 0xF, false);
}

// Inclusive scan over the 64 lanes with OP (associative; IDLE its neutral element's bit pattern): four shifted steps
// inside each row, then the row totals travel down.  Lane 63 ends with the reduction over the wave.
#define QUOKA_WAVE_SCAN(x, OP, IDLE)                                   \
  do {                                                                 \
    x = OP(x, dpp_take<0x111>(IDLE, x));                               \
    x = OP(x, dpp_take<0x112>(IDLE, x));                               \
    x = OP(x, dpp_take<0x114>(IDLE, x));                               \
    x = OP(x, dpp_take<0x118>(IDLE, x));                               \
    x = OP(x, dpp_take<0x142, 0xA>(IDLE, x));                          \
    x = OP(x, dpp_take<0x143, 0xC>(IDLE, x));                          \
  } while (0)

__device__ __forceinline__ uint32_t op_add_u32(uint32_t a, uint32_t b) { return a + b; }
__device__ __forceinline__ uint32_t op_min_u32(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ __forceinline__ uint32_t op_max_u32(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t op_add_f32(uint32_t a, uint32_t b) {
  return __float_as_uint(__uint_as_float(a) + __uint_as_float(b));
}
__device__ __forceinline__ uint32_t op_max_f32(uint32_t a, uint32_t b) {
  return __float_as_uint(fmaxf(__uint_as_float(a), __uint_as_float(b)));
}

__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t x) {
  QUOKA_WAVE_SCAN(x, op_add_u32, 0u);
  return x;
}
// Reductions over the wave; every lane gets the result (read from lane 63 into a scalar register).
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) {
  QUOKA_WAVE_SCAN(x, op_min_u32, 0xFFFFFFFFu);
  return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
  QUOKA_WAVE_SCAN(x, op_max_u32, 0u);
  return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}
__device__ __forceinline__ float wave64_sum(float xf) {
  uint32_t x = __float_as_uint(xf);
  QUOKA_WAVE_SCAN(x, op_add_f32, 0u);
  return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)x, 63));
}
__device__ __forceinline__ float wave64_max(float xf) {
  uint32_t x = __float_as_uint(xf);
  QUOKA_WAVE_SCAN(x, op_max_f32, 0xFF800000u);   // -inf
  return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)x, 63));
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
  const uint32_t inc = wave_incl_scan_u32(x);
  __syncthreads();  // protect wsum against a previous use
  if (lane == 63) wsum[w] = inc;
  __syncthreads();
  if (w == 0) {   // wave 0 scans the NT/64 wave totals
    const uint32_t t = lane < NT / 64 ? wsum[lane] : 0u;
    const uint32_t run = wave_incl_scan_u32(t);
    if (lane < NT / 64) wsum[lane] = run - t;
    if (lane == NT / 64 - 1) wsum[NT / 64] = run;
  }
  __syncthreads();
  *total = wsum[NT / 64];
  return wsum[w] + inc - x;
}

// Block-wide radix select over keys held in registers (blocks of 1024 threads, every thread calls it).
// key[j] is an order-preserving uint32 image; bit j of `valid` says whether key[j] is a real element.  Finds the key
// of the element of rank `need` (1-based; counted from the largest if DESC, else from the smallest; the caller
// guarantees need <= number of valid elements) and how many elements equal to that key belong to the first `need`.
// 8 bits per pass, starting below the leading bits that all valid keys share (scores of one head sit in a narrow
// range and would otherwise pile into one or two bins of the first passes).  One block barrier per pass: the
// histograms rotate through three LDS buffers (the buffer of pass p is cleared during pass p+2's predecessor), and
// every wave locates the cut bin for itself from the finished histogram, so nothing is handed around through LDS.
struct RadixSelectLds {
  uint32_t hist[3][256];
  uint32_t wmin[16], wmax[16];
};

template <int IPT, bool DESC>
__device__ __forceinline__ void block_radix_select(const uint32_t (&key)[IPT], uint32_t valid, uint32_t need,
                                                   RadixSelectLds& L, uint32_t* cut_key, uint32_t* need_eq) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid < 768) (&L.hist[0][0])[tid] = 0u;
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    if ((valid >> j) & 1u) {
      kmin = min(kmin, key[j]);
      kmax = max(kmax, key[j]);
    }
  }
  kmin = wave_min_u32(kmin);
  kmax = wave_max_u32(kmax);
  if (lane == 0) {
    L.wmin[w] = kmin;
    L.wmax[w] = kmax;
  }
  __syncthreads();
  kmin = wave_min_u32(lane < 16 ? L.wmin[lane] : 0xFFFFFFFFu);
  kmax = wave_max_u32(lane < 16 ? L.wmax[lane] : 0u);
  const uint32_t diff = kmin ^ kmax;
  int hi = diff ? 32 - __clz(diff) : 0;                                    // valid keys agree on all bits >= hi
  uint32_t mask = hi >= 32 ? 0u : ~((hi == 0) ? 0u : ((1u << hi) - 1u));   // decided bits
  uint32_t prefix = kmax & mask;                                           // (kmin and kmax agree there)
  uint32_t* h_use = L.hist[0];
  uint32_t* h_next = L.hist[1];
  uint32_t* h_clear = L.hist[2];
  bool first = true;
  while (hi > 0) {
    const int lo_bit = max(hi - 8, 0);
    const uint32_t dmask = (1u << (hi - lo_bit)) - 1u;
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
      const uint32_t k = key[j];
      if (((valid >> j) & 1u) && (k & mask) == prefix) atomicAdd(&h_use[(k >> lo_bit) & dmask], 1u);
    }
    __syncthreads();
    // h_clear was last read before this barrier (during the previous pass) and is next written after the next one
    if (!first && tid < 256) h_clear[tid] = 0u;
    first = false;
    // scan order position o = 4*lane + i is bin 255-o (DESC) or o
    const u32x4 raw = *reinterpret_cast<const u32x4*>(h_use + 4 * (DESC ? 63 - lane : lane));
    uint32_t c[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) c[i] = DESC ? raw[3 - i] : raw[i];
    const uint32_t sum = c[0] + c[1] + c[2] + c[3];
    const uint32_t inc = wave_incl_scan_u32(sum);
    const uint32_t excl = inc - sum;
    const bool hit = excl < need && need <= inc;   // exactly one lane
    uint32_t rem = need - excl;
    int i = 0;
#pragma unroll
    for (; i < 3; ++i) {
      if (rem <= c[i]) break;
      rem -= c[i];
    }
    const int o = 4 * lane + i;
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(hit);
    if (bal == 0) break;   // cannot happen while need <= number of valid elements
    const int src = __builtin_ctzll(bal);
    const uint32_t bin = (uint32_t)__builtin_amdgcn_readlane(DESC ? 255 - o : o, src);
    need = (uint32_t)__builtin_amdgcn_readlane((int)rem, src);
    prefix |= bin << lo_bit;
    mask |= dmask << lo_bit;
    hi = lo_bit;
    uint32_t* t = h_use;
    h_use = h_next;
    h_next = h_clear;
    h_clear = t;
  }
  *cut_key = prefix;
  *need_eq = need;
}

}  // namespace quoka
