// Chunk attention in float32 (Alg. 2 attention step; Eq. 2-3) for the float32 storage type.
// One wave per query row: lanes take 64 keys at a time for the logits, then own head_dim / 64 output
// dims each for the value accumulation; online softmax in float32.  Serves the sparse path (cache
// rows through k_idx) and the dense baseline.
#include "common.hip.h"
#include "kernels.h"

namespace quoka {

constexpr int kF32Threads = 256;

template <int D>
__global__ __launch_bounds__(kF32Threads) void attn_f32(Dims dm, AttnArgs a) {
  constexpr int EPL = D / 64;
  __shared__ float qs[kF32Threads / 64][D];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int i = blockIdx.x * (kF32Threads / 64) + w;   // chunk position of this wave's row
  const int h = blockIdx.y, b = blockIdx.z;
  const bool row_on = i < dm.C;
  if (row_on) {
    const float* qsrc = static_cast<const float*>(a.q) + b * dm.qs[0] + h * dm.qs[1] + (size_t)i * dm.qs[2];
#pragma unroll
    for (int e = 0; e < EPL; ++e) qs[w][lane + 64 * e] = qsrc[lane + 64 * e];
  }
  __syncthreads();
  if (!row_on) return;   // wave-uniform; no barrier follows
  const int kv = h / dm.g;
  const bool sparse = a.k_idx != nullptr;
  int n_cache = sparse ? min(a.n_cache[b * dm.n_kv + kv], dm.B_max) : min(a.n_cache[b], dm.T_max);
  n_cache = max(n_cache, 0);
  const int32_t* kidx = sparse ? a.k_idx + (size_t)(b * dm.n_kv + kv) * dm.B_max : nullptr;
  const float* kcache = static_cast<const float*>(a.k_cache) + b * dm.kvs[0] + kv * dm.kvs[1];
  const float* vcache = static_cast<const float*>(a.v_cache) + b * dm.kvs[0] + kv * dm.kvs[1];
  const float* kchunk = static_cast<const float*>(a.k_chunk) + b * dm.cks[0] + kv * dm.cks[1];
  const float* vchunk = static_cast<const float*>(a.v_chunk) + b * dm.cks[0] + kv * dm.cks[1];
  const float scale = 1.0f / sqrtf((float)D);
  const int total = n_cache + i + 1;
  float m_run = -INFINITY, l_run = 0.f;
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

  for (int j0 = 0; j0 < total; j0 += 64) {
    const int j = j0 + lane;
    const bool valid = j < total;
    const int jj = valid ? j : total - 1;
    int is_chunk, row;
    if (jj < n_cache) {
      is_chunk = 0;
      row = sparse ? (int)min((uint32_t)kidx[jj], (uint32_t)(dm.T_max - 1)) : jj;   // a malformed list cannot leave the cache
    } else {
      is_chunk = 1;
      row = jj - n_cache;
    }
    const float* kp = is_chunk ? kchunk + (size_t)row * dm.cks[2] : kcache + (size_t)row * dm.kvs[2];
    float dot = 0.f;
#pragma unroll 8
    for (int d0 = 0; d0 < D; d0 += 4) {
      const float4 kx = *reinterpret_cast<const float4*>(kp + d0);
      dot += qs[w][d0] * kx.x;
      dot += qs[w][d0 + 1] * kx.y;
      dot += qs[w][d0 + 2] * kx.z;
      dot += qs[w][d0 + 3] * kx.w;
    }
    const float s = valid ? dot * scale : -INFINITY;
    const float m_new = fmaxf(m_run, wave64_max(s));   // finite: key j0 is always visible
    const float alpha = expf(m_run - m_new);
    const float p = valid ? expf(s - m_new) : 0.f;
    l_run = l_run * alpha + wave64_sum(p);
    m_run = m_new;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
    const int cnt = min(64, total - j0);
    for (int t = 0; t < cnt; ++t) {
      // t is wave-uniform: lane reads through the scalar path instead of LDS shuffles
      const float pt = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(p), t));
      const int ct = __builtin_amdgcn_readlane(is_chunk, t);
      const int rt = __builtin_amdgcn_readlane(row, t);
      const float* vp = ct ? vchunk + (size_t)rt * dm.cks[2] : vcache + (size_t)rt * dm.kvs[2];
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] += pt * vp[lane + 64 * e];
    }
  }
  float* orow = static_cast<float*>(a.out) + b * dm.os[0] + h * dm.os[1] + (size_t)i * dm.os[2];
#pragma unroll
  for (int e = 0; e < EPL; ++e) orow[lane + 64 * e] = acc[e] / l_run;
  if (a.lse != nullptr && lane == 0) a.lse[(size_t)(b * dm.n_q + h) * dm.C + i] = m_run + logf(l_run);
}

hipError_t launch_attn_f32(const Dims& dm, const AttnArgs& a, hipStream_t st) {
  dim3 grid((dm.C + kF32Threads / 64 - 1) / (kF32Threads / 64), dm.n_q, dm.b);
  if (dm.d == 64) {
    hipLaunchKernelGGL((attn_f32<64>), grid, dim3(kF32Threads), 0, st, dm, a);
  } else {
    hipLaunchKernelGGL((attn_f32<128>), grid, dim3(kF32Threads), 0, st, dm, a);
  }
  return hipGetLastError();
}

}  // namespace quoka
