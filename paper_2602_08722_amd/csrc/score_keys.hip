// Key scoring (Alg. 1: K normalisation, S = Qbar K^T, S-hat = max over the query axis; Sec. 3.2-3.3).
//
// scores[b,kv,t] = max_r <Qbar[b,kv,r,:], K[b,kv,t,:]> / max(||K[b,kv,t,:]||, eps).
// The 1/||k|| factor is positive, so it is applied after the max; S itself is never stored.
//
// bf16 keys: the K cache is streamed once from HBM in 128-key tiles (coalesced 16-byte loads, double
// buffered through LDS).  Qbar (float32) is split into three bf16 terms hi + mid + lo that add up to the
// float32 value exactly, so with bf16 keys every MFMA product is exact and only the float32
// accumulation rounds.  Queries are the M side of v_mfma_f32_32x32x16_bf16, keys the N side: a lane
// owns one key column and 16 query rows, so the max over queries is in-register plus one
// half-wave exchange.
// float32 keys: plain FMA loop, one key per thread, Qbar broadcast from LDS.
#include "common.hip.h"
#include "kernels.h"

namespace quoka {

constexpr int kScThreads = 256;
constexpr int kScTile = 128;  // keys per LDS tile

template <int D, int QB>
struct ScoreCfg {
  static constexpr int KS = D / 16;             // MFMA k-steps over head_dim
  static constexpr int LD = D + 8;              // padded LDS row, elements (16-byte pad: conflict-free b128 reads)
  static constexpr int CG = D / 8;              // 16-byte chunks per key row
  static constexpr int RPI = kScThreads / CG;   // key rows covered by one block-wide load
  static constexpr int NLD = kScTile / RPI;     // loads per thread per tile
  static constexpr int KG = 4 / QB;             // wave groups that split a tile's keys
  static constexpr int KPW = kScTile / KG;      // keys per wave per tile
  static constexpr size_t kTileBytes = (size_t)kScTile * LD * 2;
  static constexpr size_t kLdsBytes = 2 * kTileBytes + 2 * kScTile * 4 + QB * kScTile * 4;
};

__device__ __forceinline__ float sumsq_bf16x8(const u32x4& r) {
  float s = 0.f;
  const uint32_t w[4] = {r[0], r[1], r[2], r[3]};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float a = __uint_as_float(w[i] << 16), b = __uint_as_float(w[i] & 0xFFFF0000u);
    s += a * a;
    s += b * b;
  }
  return s;
}

template <int D, int QB>
__global__ __launch_bounds__(kScThreads, 2) void score_bf16(Dims dm, const float* __restrict__ qbar,
                                                           const uint16_t* __restrict__ kc,
                                                           const int32_t* __restrict__ kv_lens,
                                                           float* __restrict__ scores, int n_keep, int tiles_per_wg) {
  using Cfg = ScoreCfg<D, QB>;
  constexpr int KS = Cfg::KS, LD = Cfg::LD, CG = Cfg::CG, RPI = Cfg::RPI, NLD = Cfg::NLD, KPW = Cfg::KPW;
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* tile0p = reinterpret_cast<uint16_t*>(smem);
  uint16_t* tile1p = reinterpret_cast<uint16_t*>(smem + Cfg::kTileBytes);
  float* ssq = reinterpret_cast<float*>(smem + 2 * Cfg::kTileBytes);   // [2][kScTile]
  float* smax = ssq + 2 * kScTile;                                       // [QB][kScTile]

  const int kv = blockIdx.y, b = blockIdx.z;
  const int T = min(kv_lens[b], dm.T_max);
  const int t_begin = blockIdx.x * tiles_per_wg * kScTile;
  if (t_begin >= T) return;  // block-uniform
  const int n_tiles = min(tiles_per_wg, (T - t_begin + kScTile - 1) / kScTile);

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int qb = w % QB, kg = w / QB;
  const int li = lane & 31, hf = lane >> 5;

  const uint16_t* kbase = kc + b * dm.kvs[0] + kv * dm.kvs[1];
  float* sc = scores + (size_t)(b * dm.n_kv + kv) * dm.T_max;
  const int cg = tid % CG, r0 = tid / CG;

  u32x4 R[NLD];
  auto issue = [&](int it) {
    const int t0 = t_begin + it * kScTile;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      int row = t0 + r0 + RPI * i;
      row = row < T ? row : T - 1;  // tail rows re-read the last valid key; their scores are not stored
      R[i] = *reinterpret_cast<const u32x4*>(kbase + (size_t)row * dm.kvs[2] + cg * 8);
    }
  };
  issue(0);   // the first K tile is in flight while the query operands are prepared


  // Query operands: this wave's 32 query rows, split into three bf16 terms.
  bf16x8 a_hi[KS], a_mid[KS], a_lo[KS];
  {
    int r = qb * 32 + li;
    r = r < n_keep ? r : n_keep - 1;  // padding rows repeat a real query: the max is unchanged
    const float* qrow = qbar + ((size_t)(b * dm.n_kv + kv) * n_keep + r) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const float4 x0 = *reinterpret_cast<const float4*>(qrow + ks * 16);
      const float4 x1 = *reinterpret_cast<const float4*>(qrow + ks * 16 + 4);
      const float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const __bf16 h = (__bf16)x[e];
        const float r1 = x[e] - (float)h;
        const __bf16 m = (__bf16)r1;
        const float r2 = r1 - (float)m;
        a_hi[ks][e] = h;
        a_mid[ks][e] = m;
        a_lo[ks][e] = (__bf16)r2;
      }
    }
  }

  for (int it = 0; it < n_tiles; ++it) {
    const int buf = it & 1;
    uint16_t* tl = buf ? tile1p : tile0p;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int rl = r0 + RPI * i;
      *reinterpret_cast<u32x4*>(tl + rl * LD + cg * 8) = R[i];
      float ss = sumsq_bf16x8(R[i]);
      if constexpr (CG == 16) {
        ss = row16_sum(ss);   // a key row is exactly one 16-lane DPP row
      } else {
        ss = group_sum<CG>(ss);
      }
      if (cg == 0) ssq[buf * kScTile + rl] = ss;
    }
    __syncthreads();
    if (it + 1 < n_tiles) issue(it + 1);  // next tile's HBM loads fly during the MFMA loop

#pragma unroll
    for (int kb = 0; kb < KPW / 32; ++kb) {
      const int key_l = kg * KPW + kb * 32 + li;
      const uint16_t* kp = tl + key_l * LD + 8 * hf;
      f32x16 c_hi = {0}, c_mid = {0}, c_lo = {0};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 kop = *reinterpret_cast<const bf16x8*>(kp + ks * 16);
        c_lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo[ks], kop, c_lo, 0, 0, 0);
        c_mid = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_mid[ks], kop, c_mid, 0, 0, 0);
        c_hi = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi[ks], kop, c_hi, 0, 0, 0);
      }
      float m = -INFINITY;
#pragma unroll
      for (int v = 0; v < 16; ++v) m = fmaxf(m, c_hi[v] + (c_mid[v] + c_lo[v]));
      m = fmaxf(m, other_half(m));
      if (hf == 0) smax[qb * kScTile + key_l] = m;
    }
    __syncthreads();
    if (tid < kScTile) {
      const int key = t_begin + it * kScTile + tid;
      if (key < T) {
        float m = smax[tid];
#pragma unroll
        for (int j = 1; j < QB; ++j) m = fmaxf(m, smax[j * kScTile + tid]);
        const float nrm = fmaxf(sqrtf(ssq[buf * kScTile + tid]), kNormEps);
        sc[key] = m / nrm + 0.0f;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kScThreads) void score_f32(Dims dm, const float* __restrict__ qbar,
                                                       const float* __restrict__ kc,
                                                       const int32_t* __restrict__ kv_lens, float* __restrict__ scores,
                                                       int n_keep) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* qs = reinterpret_cast<float*>(smem);  // [n_keep][D]
  const int kv = blockIdx.y, b = blockIdx.z;
  const int T = min(kv_lens[b], dm.T_max);
  if ((int)(blockIdx.x * kScThreads) >= T) return;
  const float* qsrc = qbar + (size_t)(b * dm.n_kv + kv) * n_keep * D;
  for (int i = threadIdx.x; i < n_keep * D; i += kScThreads) qs[i] = qsrc[i];
  __syncthreads();
  const int t = blockIdx.x * kScThreads + threadIdx.x;
  if (t >= T) return;
  const float* krow = kc + b * dm.kvs[0] + kv * dm.kvs[1] + (size_t)t * dm.kvs[2];
  float k[D];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < D; i += 4) {
    const float4 x = *reinterpret_cast<const float4*>(krow + i);
    k[i] = x.x; k[i + 1] = x.y; k[i + 2] = x.z; k[i + 3] = x.w;
    ss += x.x * x.x; ss += x.y * x.y; ss += x.z * x.z; ss += x.w * x.w;
  }
  float m = -INFINITY;
  for (int r = 0; r < n_keep; ++r) {
    const float* qr = qs + r * D;
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < D; ++i) dot += qr[i] * k[i];
    m = fmaxf(m, dot);
  }
  scores[(size_t)(b * dm.n_kv + kv) * dm.T_max + t] = m / fmaxf(sqrtf(ss), kNormEps) + 0.0f;
}

// ---------------------------------------------------------------------------------------------
template <int D, int QB>
static hipError_t launch_bf16(const Dims& dm, const float* qbar, const void* kc, const int32_t* kv_lens, float* scores,
                              int n_keep, hipStream_t st) {
  using Cfg = ScoreCfg<D, QB>;
  static bool attr_done = false;  // benign race: the attribute call is idempotent
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_bf16<D, QB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cfg::kLdsBytes);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int nt = (dm.T_max + kScTile - 1) / kScTile;
  const int heads = dm.b * dm.n_kv;
  const int wg_per_head = (1024 + heads - 1) / heads;
  int tpw = (nt + wg_per_head - 1) / wg_per_head;
  tpw = tpw < 1 ? 1 : (tpw > 8 ? 8 : tpw);
  dim3 grid((nt + tpw - 1) / tpw, dm.n_kv, dm.b);
  hipLaunchKernelGGL((score_bf16<D, QB>), grid, dim3(kScThreads), Cfg::kLdsBytes, st, dm, qbar,
                     static_cast<const uint16_t*>(kc), kv_lens, scores, n_keep, tpw);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_bf16_d(const Dims& dm, const float* qbar, const void* kc, const int32_t* kv_lens,
                                float* scores, int n_keep, hipStream_t st) {
  const int qblocks = (n_keep + 31) / 32;
  if (qblocks <= 1) return launch_bf16<D, 1>(dm, qbar, kc, kv_lens, scores, n_keep, st);
  if (qblocks == 2) return launch_bf16<D, 2>(dm, qbar, kc, kv_lens, scores, n_keep, st);
  return launch_bf16<D, 4>(dm, qbar, kc, kv_lens, scores, n_keep, st);
}

hipError_t launch_score_keys(const Dims& dm, int dtype, const float* qbar, const void* k_cache, const int32_t* kv_lens,
                             float* scores, hipStream_t st) {
  if (dm.T_max <= 0) return hipSuccess;
  const int n_keep = dm.n_ret < dm.C ? dm.n_ret : dm.C;
  if (dtype == QUOKA_BF16) {
    return dm.d == 64 ? launch_bf16_d<64>(dm, qbar, k_cache, kv_lens, scores, n_keep, st)
                      : launch_bf16_d<128>(dm, qbar, k_cache, kv_lens, scores, n_keep, st);
  }
  dim3 grid((dm.T_max + kScThreads - 1) / kScThreads, dm.n_kv, dm.b);
  const size_t lds = (size_t)n_keep * dm.d * sizeof(float);
  if (dm.d == 64) {
    hipLaunchKernelGGL((score_f32<64>), grid, dim3(kScThreads), lds, st, dm, qbar, static_cast<const float*>(k_cache),
                       kv_lens, scores, n_keep);
  } else {
    static bool attr_done = false;
    if (!attr_done) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_f32<128>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 128 * 4);
      if (e != hipSuccess) return e;
      attr_done = true;
    }
    hipLaunchKernelGGL((score_f32<128>), grid, dim3(kScThreads), lds, st, dm, qbar, static_cast<const float*>(k_cache),
                       kv_lens, scores, n_keep);
  }
  return hipGetLastError();
}

}  // namespace quoka
