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
#include "score_tile.hip.h"

namespace quoka {

// EXACT: Qbar enters as the three-term split (float32-exact products).  Otherwise it is rounded to bf16 once and
// only that term is multiplied: a third of the matrix work, scores within 2^-9 * sum|qbar_i| of the exact ones.
template <int D, int QB, bool EXACT>
__global__ __launch_bounds__(kScThreads, 2) void score_bf16(Dims dm, const float* __restrict__ qbar,
                                                           const uint16_t* __restrict__ kc,
                                                           const int32_t* __restrict__ kv_lens,
                                                           float* __restrict__ scores, int n_keep, int tiles_per_wg,
                                                           uint32_t* __restrict__ zero, uint32_t zero_words) {
  using Cfg = ScoreCfg<D, QB>;
  clear_words(zero, zero_words);
  constexpr int LD = Cfg::LD, CG = Cfg::CG, RPI = Cfg::RPI, NLD = Cfg::NLD;
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* tile0p = reinterpret_cast<uint16_t*>(smem);
  uint16_t* tile1p = reinterpret_cast<uint16_t*>(smem + Cfg::kTileBytes);
  float* ssq = reinterpret_cast<float*>(smem + 2 * Cfg::kTileBytes);   // [3][kScTile]
  float* smax = ssq + 3 * kScTile;                                       // [3][QB][kScTile]

  const int kv = blockIdx.y, b = blockIdx.z;
  const int t_begin = blockIdx.x * tiles_per_wg * kScTile;

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qb = w % QB, kg = w / QB;
  const int li = lane & 31, hf = lane >> 5;

  // rows of this (batch, KV head) are addressed as base + 32-bit byte offset (the host checks the 4 GiB span)
  const char* kbase = reinterpret_cast<const char*>(kc + b * dm.kvs[0] + kv * dm.kvs[1]);
  const uint32_t row_bytes = (uint32_t)dm.kvs[2] * 2u;
  float* sc = scores + (size_t)(b * dm.n_kv + kv) * dm.T_max;
  const int cg = tid % CG, r0 = tid / CG;

  // two tiles are kept in flight: even tiles travel through RA, odd tiles through RB
  u32x4 RA[NLD], RB[NLD];
  auto issue = [&](int it, u32x4 (&R)[NLD]) __attribute__((always_inline)) {
    const int t0 = t_begin + it * kScTile;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      // rows are clamped to the cache extent, not to the sequence length: loads then do not wait for the length, and
      // rows past it (allocated, arbitrary content) only produce scores that are never stored
      const int row = min(t0 + r0 + RPI * i, dm.T_max - 1);
      R[i] = *reinterpret_cast<const u32x4*>(kbase + ((uint32_t)row * row_bytes + (uint32_t)cg * 16u));
    }
  };
  issue(0, RA);   // the first K tile is in flight while the length arrives and the query operands are prepared
  const int T = min(kv_lens[b], dm.T_max);
  if (t_begin >= T) return;  // block-uniform
  const int n_tiles = min(tiles_per_wg, (T - t_begin + kScTile - 1) / kScTile);
  if (n_tiles > 1) issue(1, RB);

  const bool dot_mode = (dm.flags & 1) != 0, mean_mode = (dm.flags & 2) != 0;   // ablation scorers
  QueryTerms<D, EXACT> qt;   // this wave's 32 query rows
  qt.load(qbar + (size_t)(b * dm.n_kv + kv) * n_keep * D, n_keep, qb, li, hf, mean_mode);

  // scores of tile `it` from the maxima and squared norms of generation it % 3
  auto finish = [&](int it) {
    if (tid < kScTile) {
      const int key = t_begin + it * kScTile + tid;
      if (key < T)
        sc[key] = tile_score<QB>(smax + (it % 3) * QB * kScTile, ssq + (it % 3) * kScTile, tid, dot_mode, mean_mode,
                                 n_keep);
    }
  };

  auto tile_step = [&](int it, u32x4 (&R)[NLD]) __attribute__((always_inline)) {
    uint16_t* tl = (it & 1) ? tile1p : tile0p;
    float* ssq_g = ssq + (it % 3) * kScTile;
    float* smax_g = smax + (it % 3) * QB * kScTile;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int rl = r0 + RPI * i;
      *reinterpret_cast<u32x4*>(tl + rl * LD + cg * 8) = R[i];
      const float ss = row_sumsq<CG>(R[i]);
      if (cg == 0) ssq_g[rl] = ss;
    }
    // One barrier per tile.  It publishes tile `it` (and its squared norms) and the maxima of tile it-1.  The K tile
    // buffer written above was last read two steps ago, before the previous barrier; the norm / maximum generation
    // written in this step was last read (by finish) three steps ago, two barriers back.
    __syncthreads();
    if (it + 2 < n_tiles) issue(it + 2, R);  // the registers are free again: fetch the tile after the next
    if (it > 0) finish(it - 1);

    tile_products<D, QB, EXACT>(tl, qt, qb, kg, li, hf, mean_mode, smax_g);
  };
  for (int it = 0; it < n_tiles; it += 2) {
    tile_step(it, RA);
    if (it + 1 < n_tiles) tile_step(it + 1, RB);
  }
  __syncthreads();
  finish(n_tiles - 1);
}

// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kScThreads) void score_f32(Dims dm, const float* __restrict__ qbar,
                                                       const float* __restrict__ kc,
                                                       const int32_t* __restrict__ kv_lens, float* __restrict__ scores,
                                                       int n_keep, uint32_t* __restrict__ zero, uint32_t zero_words) {
  extern __shared__ __align__(16) unsigned char smem[];
  clear_words(zero, zero_words);
  float* qs = reinterpret_cast<float*>(smem);  // [n_keep][D]
  const int kv = blockIdx.y, b = blockIdx.z;
  const int T = min(kv_lens[b], dm.T_max);
  if ((int)(blockIdx.x * kScThreads) >= T) return;
  const float* qsrc = qbar + (size_t)(b * dm.n_kv + kv) * n_keep * D;
  const bool round_q = (dm.flags & QUOKA_SCORE_QBAR_BF16) != 0;   // reduced-precision scorer: Qbar as bf16 values
  for (int i = threadIdx.x; i < n_keep * D; i += kScThreads)
    qs[i] = round_q ? bf16_bits_to_f32(f32_to_bf16_bits(qsrc[i])) : qsrc[i];
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
  const bool dot_mode = (dm.flags & 1) != 0, mean_mode = (dm.flags & 2) != 0;   // ablation scorers
  float m = mean_mode ? 0.f : -INFINITY;
  for (int r = 0; r < n_keep; ++r) {
    const float* qr = qs + r * D;
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < D; ++i) dot += qr[i] * k[i];
    m = mean_mode ? m + dot : fmaxf(m, dot);
  }
  if (mean_mode) m /= (float)n_keep;
  scores[(size_t)(b * dm.n_kv + kv) * dm.T_max + t] = m / (dot_mode ? 1.0f : fmaxf(sqrtf(ss), kNormEps)) + 0.0f;
}

// ---------------------------------------------------------------------------------------------
template <int D, int QB, bool EXACT>
static hipError_t launch_bf16(const Dims& dm, const float* qbar, const void* kc, const int32_t* kv_lens, float* scores,
                              int n_keep, hipStream_t st, uint32_t* zero, uint32_t zero_words) {
  using Cfg = ScoreCfg<D, QB>;
  static std::atomic<uint64_t> lds_done{0};
  const hipError_t e =
      ensure_dynamic_lds(reinterpret_cast<const void*>(&score_bf16<D, QB, EXACT>), Cfg::kLdsBytes, lds_done);
  if (e != hipSuccess) return e;
  const int nt = (dm.T_max + kScTile - 1) / kScTile;
  const int heads = dm.b * dm.n_kv;
  // two blocks per compute unit are resident at once: aim for one round of 512 blocks, so the query operands
  // (prepared once per block) are amortised over as many tiles as the launch allows
  const int wg_per_head = (512 + heads - 1) / heads;
  int tpw = (nt + wg_per_head - 1) / wg_per_head;
  tpw = tpw < 1 ? 1 : tpw;
  dim3 grid((nt + tpw - 1) / tpw, dm.n_kv, dm.b);
  hipLaunchKernelGGL((score_bf16<D, QB, EXACT>), grid, dim3(kScThreads), Cfg::kLdsBytes, st, dm, qbar,
                     static_cast<const uint16_t*>(kc), kv_lens, scores, n_keep, tpw, zero, zero_words);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_bf16_d(const Dims& dm, const float* qbar, const void* kc, const int32_t* kv_lens,
                                float* scores, int n_keep, hipStream_t st, uint32_t* zero, uint32_t zero_words) {
  const int qblocks = (n_keep + 31) / 32;
  if (dm.flags & QUOKA_SCORE_QBAR_BF16) {
    if (qblocks <= 1) return launch_bf16<D, 1, false>(dm, qbar, kc, kv_lens, scores, n_keep, st, zero, zero_words);
    if (qblocks == 2) return launch_bf16<D, 2, false>(dm, qbar, kc, kv_lens, scores, n_keep, st, zero, zero_words);
    return launch_bf16<D, 4, false>(dm, qbar, kc, kv_lens, scores, n_keep, st, zero, zero_words);
  }
  if (qblocks <= 1) return launch_bf16<D, 1, true>(dm, qbar, kc, kv_lens, scores, n_keep, st, zero, zero_words);
  if (qblocks == 2) return launch_bf16<D, 2, true>(dm, qbar, kc, kv_lens, scores, n_keep, st, zero, zero_words);
  return launch_bf16<D, 4, true>(dm, qbar, kc, kv_lens, scores, n_keep, st, zero, zero_words);
}

hipError_t launch_score_keys(const Dims& dm, int dtype, const float* qbar, const void* k_cache, const int32_t* kv_lens,
                             float* scores, hipStream_t st, uint32_t* zero, size_t zero_words_sz) {
  if (dm.T_max <= 0) return hipSuccess;   // (then the top-k that follows takes no workspace either)
  const uint32_t zero_words = (uint32_t)zero_words_sz;
  const int n_keep = dm.n_ret < dm.C ? dm.n_ret : dm.C;
  if (dtype == QUOKA_BF16) {
    return dm.d == 64 ? launch_bf16_d<64>(dm, qbar, k_cache, kv_lens, scores, n_keep, st, zero, zero_words)
                      : launch_bf16_d<128>(dm, qbar, k_cache, kv_lens, scores, n_keep, st, zero, zero_words);
  }
  dim3 grid((dm.T_max + kScThreads - 1) / kScThreads, dm.n_kv, dm.b);
  const size_t lds = (size_t)n_keep * dm.d * sizeof(float);
  if (dm.d == 64) {
    hipLaunchKernelGGL((score_f32<64>), grid, dim3(kScThreads), lds, st, dm, qbar, static_cast<const float*>(k_cache),
                       kv_lens, scores, n_keep, zero, zero_words);
  } else {
    static std::atomic<uint64_t> lds_done{0};
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&score_f32<128>), 128 * 128 * 4, lds_done);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((score_f32<128>), grid, dim3(kScThreads), lds, st, dm, qbar, static_cast<const float*>(k_cache),
                       kv_lens, scores, n_keep, zero, zero_words);
  }
  return hipGetLastError();
}

}  // namespace quoka
