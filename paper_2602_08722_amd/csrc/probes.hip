// Measurement aids: three kernels of known work that a benchmark times next to the library's own kernels, so that
// a kernel's rate can be quoted against what this GPU sustains (at the clock it actually runs at) as well as
// against the published peaks.
//   probe_mfma : register-only chains of v_mfma_f32_32x32x16_bf16, two waves per SIMD, no memory traffic.
//   probe_read : every byte of a buffer read once with coalesced 16-byte loads, nothing written.
//   probe_attn_mix : the instruction mix of the attention kernel's step without its memory side -- per wave and
//                step 16 MFMAs in two chains (S = K Q^T), then 32 exponentials and about 160 plain vector
//                operations (scaling, max, conversion to bf16) interleaved with 16 MFMAs in four chains (O += P V);
//                eight waves per compute unit, no LDS traffic, no barriers.  What it reaches is the ceiling of any
//                kernel that keeps this work split (32 query rows per wave, two waves per SIMD).
#include "common.hip.h"
#include "kernels.h"

namespace quoka {

constexpr int kProbeThreads = 256;

__global__ __launch_bounds__(kProbeThreads, 2) void probe_mfma(int iters, float* __restrict__ sink) {
  // operands from the lane id: finite, small, different per lane (their values do not matter)
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(0.001f * (float)((threadIdx.x + e) & 31));
    b[e] = (__bf16)(0.002f * (float)((threadIdx.x * 3 + e) & 15));
  }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};   // four independent chains hide the MFMA result latency
  for (int i = 0; i < iters; ++i) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int v = 0; v < 16; ++v) s += c0[v] + c1[v] + c2[v] + c3[v];
  if (s == -1.0f) sink[0] = s;   // never true (all products are >= 0): keeps the chains alive
}

__global__ __launch_bounds__(kProbeThreads) void probe_read(const u32x4* __restrict__ src, size_t n16,
                                                          float* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * kProbeThreads;
  size_t i = (size_t)blockIdx.x * kProbeThreads + threadIdx.x;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + 7 * stride < n16; i += 8 * stride) {   // eight loads in flight per thread
    u32x4 r[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) r[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= r[u];
  }
  for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
  // a store nobody expects to happen (it would need all four xor sums to be this pattern): keeps the loads alive
  if (acc[0] == 0x9E3779B9u && acc[1] == 0x7F4A7C15u && acc[2] == 0xF39CC060u && acc[3] == 0x5CEDC834u)
    sink[0] = 1.0f;
}

__global__ __launch_bounds__(512, 2) void probe_attn_mix(int steps, float* __restrict__ sink) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(0.01f * (float)((threadIdx.x + e) & 31));
    b[e] = (__bf16)(0.02f * (float)((threadIdx.x * 3 + e) & 15));
  }
  f32x16 s0 = {0}, s1 = {0}, o0 = {0}, o1 = {0}, o2 = {0}, o3 = {0};
  float m = 0.f;
  for (int it = 0; it < steps; ++it) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, ks == 0 ? f32x16{0} : s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, ks == 0 ? f32x16{0} : s1, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float x = s0[v], y = s1[v];
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        x = fmaf(x, 0.999f, m);
        y = fmaf(y, 0.999f, -m);
      }
      x = __builtin_amdgcn_exp2f(x);
      y = __builtin_amdgcn_exp2f(y);
      m = fmaxf(m * 0.5f, x - y);
      bf16x8 pb;
#pragma unroll
      for (int e = 0; e < 8; ++e) pb[e] = (__bf16)((e & 1) ? x : y);
      if ((v & 3) == 0) o0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, o0, 0, 0, 0);
      if ((v & 3) == 1) o1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, o1, 0, 0, 0);
      if ((v & 3) == 2) o2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, o2, 0, 0, 0);
      if ((v & 3) == 3) o3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, o3, 0, 0, 0);
    }
  }
  float t = m;
#pragma unroll
  for (int v = 0; v < 16; ++v) t += o0[v] + o1[v] + o2[v] + o3[v] + s0[v] + s1[v];
  if (t == -12345.f) sink[0] = t;   // never true in practice: keeps the work alive
}

hipError_t launch_probe_attn_mix(int blocks, int steps, float* sink, hipStream_t st) {
  hipLaunchKernelGGL(probe_attn_mix, dim3(blocks), dim3(512), 0, st, steps, sink);
  return hipGetLastError();
}

hipError_t launch_probe_mfma(int blocks, int iters, float* sink, hipStream_t st) {
  hipLaunchKernelGGL(probe_mfma, dim3(blocks), dim3(kProbeThreads), 0, st, iters, sink);
  return hipGetLastError();
}

hipError_t launch_probe_read(const void* src, size_t bytes, float* sink, hipStream_t st) {
  // 2048 blocks of 256 threads x 8 loads x 16 bytes = 64 MiB per sweep of the grid
  hipLaunchKernelGGL(probe_read, dim3(2048), dim3(kProbeThreads), 0, st, static_cast<const u32x4*>(src), bytes / 16,
                     sink);
  return hipGetLastError();
}

}  // namespace quoka
