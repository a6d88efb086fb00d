// Key scoring and top-B selection as one stage for long caches (Alg. 1: S = Qbar K^T, S-hat = max, I = topk(S-hat,
// B_SA); the paper's conclusion names a cheaper Qbar K^T as the thing to improve).
//
// The exact product costs three bf16 MFMA terms per key (Qbar is float32).  Only the keys near the cut need it:
//   1. provisional scores p from ONE term (Qbar rounded to bf16).  For every key |p - s| <= eps, where s is the exact
//      score and eps = max_r ||qbar_r - bf16(qbar_r)||_2 (Cauchy-Schwarz with the unit key; the max over queries moves
//      by at most the largest per-query error), plus the float32 accumulation slack of both;
//   2. a histogram of p over 4096 equal bins of [-1, 1] locates the bin of the provisional cut (the B-th largest p);
//   3. keys whose bin lies more than m bins above the cut bin are certainly selected, keys more than m bins below it
//      certainly not (m bins cover 2 eps and the width of the cut bin); the keys in between -- the band, a few per
//      cent -- are scored again with the exact three-term product, by the same tile arithmetic as the streaming
//      kernel, so their scores carry the same float32 bits;
//   4. the best (B - certain) band keys by exact score complete the set; equal scores go to the lower position;
//      indices come out in ascending position.
// The selected set is therefore exactly the top-B of the exact scores, as the separate scoring and top-B calls
// produce it; the `scores` array ends up holding exact values inside the band and provisional values elsewhere.
//
// Launch chain (no block ever waits for another block of its launch): provisional scoring, histogram, band
// classification + exact re-scoring per 2048-key tile, one block per head that selects among the band candidates
// and lays out the tiles' output offsets, ordered emission per tile.
#include "common.hip.h"
#include "kernels.h"
#include "score_tile.hip.h"

namespace quoka {

constexpr int kSelBins = 4096;        // equal bins over [-1, 1]
constexpr int kSelTile = 2048;        // keys per block in the per-tile kernels
constexpr int kSelThreads = 256;
constexpr int kSelIPT = kSelTile / kSelThreads;
constexpr int kSelMeta = 16;          // per-head words: candidate count, band limits, exact cut
constexpr int kSelHeadThreads = 1024;
constexpr int kSelMaxTiles = (1 << 24) / kSelTile;   // the interface limits a cache to 2^24 - 1 positions

enum { kMetaCand = 0, kMetaBinLo = 1, kMetaBinHi = 2, kMetaTau = 3, kMetaNeedEq = 4 };

// Bin of a provisional score: monotone in p, the same expression wherever it is evaluated.
__device__ __forceinline__ int score_bin(float p) {
  const float x = (p + 1.0f) * (float)(kSelBins / 2);
  return min(max((int)floorf(x), 0), kSelBins - 1);
}

// Workspace of the stage.  The words that must be zero when the chain starts (histograms and candidate counters of
// all heads) come first, in one contiguous run, so that an earlier launch can clear them as a side job.
struct SelWs {
  uint32_t *hist, *meta, *tile_in, *tile_off, *tile_eqb, *mask, *cand_key, *cand_pos;
};
__host__ __device__ inline int sel_tiles(int T_max) { return (T_max + kSelTile - 1) / kSelTile; }
__host__ __device__ inline size_t sel_mask_words(int T_max) { return (size_t)sel_tiles(T_max) * (kSelTile / 32); }
__host__ __device__ inline size_t sel_zero_words(int heads) { return (size_t)heads * (kSelBins + kSelMeta); }
__host__ __device__ inline size_t sel_head_words(int T_max) {
  return 3 * (size_t)sel_tiles(T_max) + sel_mask_words(T_max) + 2 * (size_t)T_max;
}
__device__ __forceinline__ SelWs sel_ws(uint32_t* ws, int heads, int head, int T_max) {
  SelWs s;
  s.hist = ws + (size_t)head * (kSelBins + kSelMeta);
  s.meta = s.hist + kSelBins;
  uint32_t* p = ws + sel_zero_words(heads) + (size_t)head * sel_head_words(T_max);
  const int nt = sel_tiles(T_max);
  s.tile_in = p;
  s.tile_off = p + nt;
  s.tile_eqb = p + 2 * nt;
  s.mask = p + 3 * nt;
  s.cand_key = s.mask + sel_mask_words(T_max);
  s.cand_pos = s.cand_key + T_max;
  return s;
}

struct SelCtx {
  int T, B, head;
  float* sc;
  SelWs w;
};
__device__ __forceinline__ SelCtx sel_ctx(const Dims& dm, float* scores, const int32_t* kv_lens,
                                          const int32_t* budgets, uint32_t* ws, int kv, int b) {
  SelCtx c;
  c.T = max(0, min(kv_lens[b], dm.T_max));
  c.B = max(0, min(min(budgets[b], c.T), dm.B_max));
  c.head = b * dm.n_kv + kv;
  c.sc = scores + (size_t)c.head * dm.T_max;
  c.w = sel_ws(ws, dm.b * dm.n_kv, c.head, dm.T_max);
  return c;
}

__global__ void sel_zero(uint32_t* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// ---------------------------------------------------------------------------------------------
// Histogram of the provisional scores of one tile (LDS histogram, integer-atomic flush of the occupied bins).
__global__ __launch_bounds__(kSelThreads) void sel_hist(Dims dm, float* __restrict__ scores,
                                                       const int32_t* __restrict__ kv_lens,
                                                       const int32_t* __restrict__ budgets, uint32_t* __restrict__ ws) {
  __shared__ uint32_t lh[kSelBins];
  const SelCtx c = sel_ctx(dm, scores, kv_lens, budgets, ws, blockIdx.y, blockIdx.z);
  const int t0 = blockIdx.x * kSelTile;
  if (c.B == 0 || c.B >= c.T || t0 >= c.T) return;   // block-uniform: nothing to select, or everything
  for (int i = threadIdx.x; i < kSelBins; i += kSelThreads) lh[i] = 0u;
  __syncthreads();
  const int t1 = min(t0 + kSelTile, c.T);
  for (int t = t0 + threadIdx.x; t < t1; t += kSelThreads) atomicAdd(&lh[score_bin(c.sc[t])], 1u);
  __syncthreads();
  for (int i = threadIdx.x; i < kSelBins; i += kSelThreads) {
    const uint32_t v = lh[i];
    if (v) atomicAdd(&c.w.hist[i], v);
  }
}

// ---------------------------------------------------------------------------------------------
// Per tile: locate the band from the finished histogram, classify the tile's keys, score the band keys exactly.
template <int D, int QB>
__global__ __launch_bounds__(kSelThreads) void sel_band_rescore(Dims dm, const float* __restrict__ qbar,
                                                               const uint16_t* __restrict__ kc,
                                                               const int32_t* __restrict__ kv_lens,
                                                               const int32_t* __restrict__ budgets,
                                                               float* __restrict__ scores, uint32_t* __restrict__ ws,
                                                               int n_keep) {
  using Cfg = ScoreCfg<D, QB>;
  constexpr int LD = Cfg::LD, CG = Cfg::CG, RPI = Cfg::RPI, NLD = Cfg::NLD;
  __shared__ __align__(16) uint16_t tile[kScTile * LD];
  __shared__ float ssq[kScTile];
  __shared__ float smax[QB * kScTile];
  __shared__ uint32_t band_loc[kSelTile];        // positions (relative to the tile) of the band keys, any order
  __shared__ uint32_t sh[kSelThreads + 2];
  __shared__ float red[kSelThreads / 64];
  __shared__ uint32_t bc[4];                     // cut bin, band count, sure-in count, candidate slot base

  const int kv = blockIdx.y, b = blockIdx.z;
  const SelCtx c = sel_ctx(dm, scores, kv_lens, budgets, ws, kv, b);
  const int t0 = blockIdx.x * kSelTile;
  if (c.B == 0 || c.B >= c.T || t0 >= c.T) return;   // block-uniform
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (tid < 4) bc[tid] = 0u;

  // provisional scores of the tile, requested before anything else (position t0 + tid + 256 * i: coalesced rows)
  float p[kSelIPT];
#pragma unroll
  for (int i = 0; i < kSelIPT; ++i) {
    const int t = t0 + tid + kSelThreads * i;
    p[i] = t < c.T ? c.sc[t] : 0.f;
  }

  // ---- the bin of the provisional cut: scanning from the top, where the running count reaches B ----
  {
    constexpr uint32_t per = kSelBins / kSelThreads;
    const uint32_t top = kSelBins - tid * per;   // exclusive upper bin of this thread's run (thread 0: highest bins)
    uint32_t hv[per];
#pragma unroll
    for (uint32_t i = 0; i < per; i += 4) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(c.w.hist + top - per + i);
      hv[i] = v[0]; hv[i + 1] = v[1]; hv[i + 2] = v[2]; hv[i + 3] = v[3];
    }
    uint32_t mine = 0;
#pragma unroll
    for (uint32_t i = 0; i < per; ++i) mine += hv[i];
    uint32_t tot;
    const uint32_t above = block_excl_scan<kSelThreads>(mine, sh, &tot);
    const uint32_t need = (uint32_t)c.B;
    if (above < need && need <= above + mine) {   // exactly one thread (the histogram holds T > B keys)
      uint32_t rem = need - above;
      int found = -1;
#pragma unroll
      for (int j = (int)per - 1; j >= 0; --j) {   // from this thread's highest bin down
        if (found < 0) {
          if (rem <= hv[j]) {
            found = j;
          } else {
            rem -= hv[j];
          }
        }
      }
      bc[0] = top - per + (uint32_t)max(found, 0);
    }
  }

  // ---- eps: the largest distance between a row of Qbar and its bf16 rounding ----
  float d2 = 0.f;
  {
    const float* qh = qbar + (size_t)c.head * n_keep * D;
    const int cgq = tid % CG, rq = tid / CG;
    for (int r0 = 0; r0 < n_keep; r0 += kSelThreads / CG) {   // uniform trip count; rows past the end repeat the last
      const int r = min(r0 + rq, n_keep - 1);
      const float4 x0 = *reinterpret_cast<const float4*>(qh + (size_t)r * D + cgq * 8);
      const float4 x1 = *reinterpret_cast<const float4*>(qh + (size_t)r * D + cgq * 8 + 4);
      const float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float dlt = x[e] - (float)(__bf16)x[e];
        s += dlt * dlt;
      }
      if constexpr (CG == 16) {
        s = row16_sum(s);
      } else {
        s = group_sum<CG>(s);
      }
      d2 = fmaxf(d2, s);
    }
    d2 = wave64_max(d2);
    if (lane == 0) red[w] = d2;
  }
  __syncthreads();
  d2 = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  // |p - s| <= ||delta|| (exact arithmetic) + float32 accumulation and bin-edge slack of the two computed values
  const float eps = sqrtf(d2) * 1.001f + 4e-6f;
  const int m = (int)ceilf(2.0f * eps * (float)(kSelBins / 2)) + 1;
  const int cut_bin = (int)bc[0];
  const int bin_lo = max(cut_bin - m, 0), bin_hi = min(cut_bin + m, kSelBins - 1);
  if (blockIdx.x == 0 && tid == 0) {
    c.w.meta[kMetaBinLo] = (uint32_t)bin_lo;
    c.w.meta[kMetaBinHi] = (uint32_t)bin_hi;
  }

  // ---- classify: certainly selected (counted), band (listed, flagged in the mask), certainly not ----
  uint32_t n_in = 0;
#pragma unroll
  for (int i = 0; i < kSelIPT; ++i) {
    const int tl = tid + kSelThreads * i;
    const bool valid = t0 + tl < c.T;
    const int bin = score_bin(p[i]);
    const bool inb = valid && bin >= bin_lo && bin <= bin_hi;
    n_in += (valid && bin > bin_hi) ? 1u : 0u;
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(inb);
    // positions tl of one wave in one round are 64 consecutive keys: its ballot is two words of the tile's mask
    if (lane == 0) {
      uint32_t* mw = c.w.mask + (size_t)blockIdx.x * (kSelTile / 32) + (kSelThreads * i + 64 * w) / 32;
      mw[0] = (uint32_t)bal;
      mw[1] = (uint32_t)(bal >> 32);
    }
    uint32_t base = 0;
    if (lane == 0 && bal != 0) base = atomicAdd(&bc[1], (uint32_t)__popcll(bal));
    base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
    if (inb) band_loc[base + __popcll(bal & ((1ull << lane) - 1ull))] = (uint32_t)tl;
  }
  n_in = wave_incl_scan_u32(n_in);
  if (lane == 63 && n_in) atomicAdd(&bc[2], n_in);
  __syncthreads();
  const int n_band = (int)bc[1];
  if (tid == 0) {
    c.w.tile_in[blockIdx.x] = bc[2];
    if (n_band > 0) bc[3] = atomicAdd(&c.w.meta[kMetaCand], (uint32_t)n_band);   // slots in the head's candidate list
  }
  if (n_band == 0) return;   // block-uniform
  __syncthreads();
  const uint32_t slot0 = bc[3];

  // ---- exact scores of the band keys, 128 at a time, by the tile arithmetic of the streaming kernel ----
  const int qb = w % QB, kg = w / QB;
  const int li = lane & 31, hf = lane >> 5;
  QueryTerms<D, true> qt;
  qt.load(qbar + (size_t)c.head * n_keep * D, n_keep, qb, li, hf, false);
  const char* kbase = reinterpret_cast<const char*>(kc + b * dm.kvs[0] + kv * dm.kvs[1]);
  const uint32_t row_bytes = (uint32_t)dm.kvs[2] * 2u;
  const int cg = tid % CG, r0 = tid / CG;
  for (int j0 = 0; j0 < n_band; j0 += kScTile) {
    u32x4 R[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int j = min(j0 + r0 + RPI * i, n_band - 1);   // tail slots repeat a real row; their scores are not used
      const uint32_t row = (uint32_t)t0 + band_loc[j];
      R[i] = *reinterpret_cast<const u32x4*>(kbase + (row * row_bytes + (uint32_t)cg * 16u));
    }
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int rl = r0 + RPI * i;
      *reinterpret_cast<u32x4*>(tile + rl * LD + cg * 8) = R[i];
      const float ss = row_sumsq<CG>(R[i]);
      if (cg == 0) ssq[rl] = ss;
    }
    __syncthreads();
    tile_products<D, QB, true>(tile, qt, qb, kg, li, hf, false, smax);
    __syncthreads();
    if (tid < kScTile && j0 + tid < n_band) {
      const float s = tile_score<QB>(smax, ssq, tid, false, false, n_keep);
      const uint32_t pos = (uint32_t)t0 + band_loc[j0 + tid];
      c.sc[pos] = s;
      c.w.cand_key[slot0 + j0 + tid] = max(okey(s), 1u);
      c.w.cand_pos[slot0 + j0 + tid] = pos;
    }
    __syncthreads();   // the tile, norms and maxima are overwritten by the next batch
  }
}

// ---------------------------------------------------------------------------------------------
// One block per head: the exact cut among the band candidates, then the output offset of every tile.
// Radix select (descending) over keys that are read again from memory in every pass (the candidate list of a head is
// a few tens of KiB and stays in cache; there is no bound on its length, so registers cannot hold it in general).
struct HeadSelectLds {
  uint32_t hist[3][256];
  uint32_t wmin[16], wmax[16];
  uint32_t wsum[kSelHeadThreads / 64 + 1];
};

__device__ __forceinline__ void stream_radix_select_desc(const uint32_t* __restrict__ keys, uint32_t n, uint32_t need,
                                                         HeadSelectLds& L, uint32_t* cut_key, uint32_t* need_eq) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid < 768) (&L.hist[0][0])[tid] = 0u;
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
  for (uint32_t i = tid; i < n; i += kSelHeadThreads) {
    const uint32_t k = keys[i];
    kmin = min(kmin, k);
    kmax = max(kmax, k);
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
  int hi = diff ? 32 - __clz(diff) : 0;                                    // the keys agree on all bits >= hi
  uint32_t mask = hi >= 32 ? 0u : ~((hi == 0) ? 0u : ((1u << hi) - 1u));   // decided bits
  uint32_t prefix = kmax & mask;
  uint32_t* h_use = L.hist[0];
  uint32_t* h_next = L.hist[1];
  uint32_t* h_clear = L.hist[2];
  bool first = true;
  while (hi > 0) {
    const int lo_bit = max(hi - 8, 0);
    const uint32_t dmask = (1u << (hi - lo_bit)) - 1u;
    for (uint32_t i = tid; i < n; i += kSelHeadThreads) {
      const uint32_t k = keys[i];
      if ((k & mask) == prefix) atomicAdd(&h_use[(k >> lo_bit) & dmask], 1u);
    }
    __syncthreads();
    // h_clear was last read before this barrier (during the previous pass) and is next written after the next one
    if (!first && tid < 256) h_clear[tid] = 0u;
    first = false;
    // every wave locates the cut bin for itself; scan position o = 4 * lane + i is bin 255 - o
    const u32x4 raw = *reinterpret_cast<const u32x4*>(h_use + 4 * (63 - lane));
    const uint32_t cc[4] = {raw[3], raw[2], raw[1], raw[0]};
    const uint32_t sum = cc[0] + cc[1] + cc[2] + cc[3];
    const uint32_t inc = wave_incl_scan_u32(sum);
    const uint32_t excl = inc - sum;
    const bool hit = excl < need && need <= inc;   // exactly one lane
    uint32_t rem = need - excl;
    int i = 0;
#pragma unroll
    for (; i < 3; ++i) {
      if (rem <= cc[i]) break;
      rem -= cc[i];
    }
    const int o = 4 * lane + i;
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(hit);
    if (bal == 0) break;   // cannot happen while need <= n
    const int src = __builtin_ctzll(bal);
    const uint32_t bin = (uint32_t)__builtin_amdgcn_readlane(255 - o, src);
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

__global__ __launch_bounds__(kSelHeadThreads) void sel_band_select(Dims dm, float* __restrict__ scores,
                                                                   const int32_t* __restrict__ kv_lens,
                                                                   const int32_t* __restrict__ budgets,
                                                                   uint32_t* __restrict__ ws) {
  __shared__ HeadSelectLds L;
  __shared__ uint32_t cnt[kSelMaxTiles];   // per tile: band keys above the exact cut (high half), equal to it (low half)
  const SelCtx c = sel_ctx(dm, scores, kv_lens, budgets, ws, blockIdx.x, blockIdx.y);
  if (c.B == 0 || c.B >= c.T) return;   // block-uniform
  const int tid = threadIdx.x;
  const int nt = (c.T + kSelTile - 1) / kSelTile;   // tiles of this head that the per-tile kernels worked on
  // keys that are certainly selected: everything in the bins above the band
  const uint32_t bin_hi = c.w.meta[kMetaBinHi];
  uint32_t n_in = 0;
  for (uint32_t i = bin_hi + 1 + tid; i < (uint32_t)kSelBins; i += kSelHeadThreads) n_in += c.w.hist[i];
  uint32_t tot_in;
  block_excl_scan<kSelHeadThreads>(n_in, L.wsum, &tot_in);
  const uint32_t n_c = c.w.meta[kMetaCand];
  const uint32_t need = (uint32_t)c.B - tot_in;   // >= 1: fewer than B keys lie above the cut bin, let alone the band
  for (int i = tid; i < nt; i += kSelHeadThreads) cnt[i] = 0u;
  __syncthreads();
  uint32_t tau, need_eq;
  stream_radix_select_desc(c.w.cand_key, n_c, need, L, &tau, &need_eq);
  for (uint32_t i = tid; i < n_c; i += kSelHeadThreads) {
    const uint32_t k = c.w.cand_key[i];
    if (k >= tau) atomicAdd(&cnt[c.w.cand_pos[i] / kSelTile], k > tau ? 0x10000u : 1u);
  }
  __syncthreads();
  // Output offsets.  Thread t owns tiles t*tpt .. +tpt; first the number of cut-equal band keys before every tile
  // (equal scores go to the lower positions, so a tile takes what is left of need_eq when its turn comes), then the
  // number of selected keys before it.
  const int tpt = (nt + kSelHeadThreads - 1) / kSelHeadThreads;
  const int i0 = tid * tpt, i1 = min(i0 + tpt, nt);
  uint32_t e_sum = 0;
  for (int i = i0; i < i1; ++i) e_sum += cnt[i] & 0xFFFFu;
  uint32_t tot;
  uint32_t eqb = block_excl_scan<kSelHeadThreads>(e_sum, L.wsum, &tot);
  uint32_t s_sum = 0;
  for (int i = i0; i < i1; ++i) {
    const uint32_t eq = cnt[i] & 0xFFFFu, gt = cnt[i] >> 16;
    const uint32_t take_eq = min(eq, need_eq > eqb ? need_eq - eqb : 0u);
    c.w.tile_eqb[i] = eqb;
    eqb += eq;
    const uint32_t sel = c.w.tile_in[i] + gt + take_eq;
    cnt[i] = sel;   // (own tiles only: nobody else reads them again)
    s_sum += sel;
  }
  uint32_t off = block_excl_scan<kSelHeadThreads>(s_sum, L.wsum, &tot);
  for (int i = i0; i < i1; ++i) {
    c.w.tile_off[i] = off;
    off += cnt[i];
  }
  if (tid == 0) {
    c.w.meta[kMetaTau] = tau;
    c.w.meta[kMetaNeedEq] = need_eq;
  }
}

// ---------------------------------------------------------------------------------------------
// Ordered emission per tile: thread t owns 8 consecutive positions.
__global__ __launch_bounds__(kSelThreads) void sel_emit(Dims dm, float* __restrict__ scores,
                                                       const int32_t* __restrict__ kv_lens,
                                                       const int32_t* __restrict__ budgets, uint32_t* __restrict__ ws,
                                                       int32_t* __restrict__ k_idx, int32_t* __restrict__ k_cnt) {
  __shared__ uint32_t sh[kSelThreads + 2];
  const int kv = blockIdx.y, b = blockIdx.z;
  const SelCtx c = sel_ctx(dm, scores, kv_lens, budgets, ws, kv, b);
  const int t0 = blockIdx.x * kSelTile;
  int32_t* out = k_idx + (size_t)c.head * dm.B_max;
  if (blockIdx.x == 0 && threadIdx.x == 0) k_cnt[c.head] = c.B;
  if (c.B == 0 || t0 >= c.T) return;
  const int t1 = min(t0 + kSelTile, c.T);
  if (c.B >= c.T) {
    for (int i = t0 + threadIdx.x; i < t1; i += kSelThreads) out[i] = i;
    return;
  }
  const int bin_hi = (int)c.w.meta[kMetaBinHi];
  const uint32_t tau = c.w.meta[kMetaTau], need_eq = c.w.meta[kMetaNeedEq];
  const int lo = t0 + threadIdx.x * kSelIPT;
  // this thread's 8 positions are one byte of the tile's band mask
  const uint32_t mword = c.w.mask[(size_t)blockIdx.x * (kSelTile / 32) + (threadIdx.x * kSelIPT) / 32];
  const uint32_t mbits = (mword >> ((threadIdx.x * kSelIPT) % 32)) & 0xFFu;
  uint32_t take = 0, eqm = 0;   // per position: selected regardless of ties / band key equal to the cut
  uint32_t cntp = 0;
#pragma unroll
  for (int i = 0; i < kSelIPT; ++i) {
    const int t = lo + i;
    if (t < t1) {
      const float v = c.sc[t];
      if ((mbits >> i) & 1u) {
        const uint32_t k = max(okey(v), 1u);
        take |= (k > tau ? 1u : 0u) << i;
        eqm |= (k == tau ? 1u : 0u) << i;
      } else {
        take |= (score_bin(v) > bin_hi ? 1u : 0u) << i;
      }
    }
  }
  cntp = ((uint32_t)__popc(take) << 16) | (uint32_t)__popc(eqm);
  uint32_t tot;
  const uint32_t before = block_excl_scan<kSelThreads>(cntp, sh, &tot);
  // cut-equal band keys at lower positions: in earlier tiles, then in earlier threads of this tile
  uint32_t p_eq = c.w.tile_eqb[blockIdx.x] + (before & 0xFFFFu);
  // selected keys at lower positions: earlier tiles, this tile's certain ones, and the cut-equal ones still in budget
  const uint32_t eq_tile0 = c.w.tile_eqb[blockIdx.x];
  const uint32_t taken_eq_before = min(p_eq, need_eq) - min(eq_tile0, need_eq);
  uint32_t pos = c.w.tile_off[blockIdx.x] + (before >> 16) + taken_eq_before;
#pragma unroll
  for (int i = 0; i < kSelIPT; ++i) {
    bool sel = (take >> i) & 1u;
    if ((eqm >> i) & 1u) {
      sel = p_eq < need_eq;
      ++p_eq;
    }
    if (sel) {
      if (pos < (uint32_t)c.B) out[pos] = lo + i;   // guard: inconsistent inputs cannot push writes past the budget
      ++pos;
    }
  }
}

// ---------------------------------------------------------------------------------------------
bool select_keys_two_pass_applies(const Dims& dm, int dtype) {
  // the error bound of the provisional pass is uniform only for cosine scores reduced by max; short caches take one
  // single-block top-k launch after the exact scores, which the longer chain of this stage cannot beat
  return dtype == QUOKA_BF16 && dm.T_max > 32768 &&
         (dm.flags & (QUOKA_SCORE_DOT | QUOKA_SCORE_MEAN | QUOKA_SCORE_QBAR_BF16)) == 0;
}

size_t select_keys_ws_words(const Dims& dm) {
  if (dm.T_max <= 32768) return 0;
  return sel_zero_words(dm.b * dm.n_kv) + (size_t)dm.b * dm.n_kv * sel_head_words(dm.T_max);
}

size_t select_keys_zero_words(const Dims& dm) { return sel_zero_words(dm.b * dm.n_kv); }

template <int D>
static void launch_rescore(const Dims& dm, const float* qbar, const void* kc, const int32_t* kv_lens,
                           const int32_t* budgets, float* scores, uint32_t* ws, int n_keep, dim3 grid,
                           hipStream_t st) {
  const int qblocks = (n_keep + 31) / 32;
  const uint16_t* k = static_cast<const uint16_t*>(kc);
  if (qblocks <= 1) {
    hipLaunchKernelGGL((sel_band_rescore<D, 1>), grid, dim3(kSelThreads), 0, st, dm, qbar, k, kv_lens, budgets, scores,
                       ws, n_keep);
  } else if (qblocks == 2) {
    hipLaunchKernelGGL((sel_band_rescore<D, 2>), grid, dim3(kSelThreads), 0, st, dm, qbar, k, kv_lens, budgets, scores,
                       ws, n_keep);
  } else {
    hipLaunchKernelGGL((sel_band_rescore<D, 4>), grid, dim3(kSelThreads), 0, st, dm, qbar, k, kv_lens, budgets, scores,
                       ws, n_keep);
  }
}

hipError_t launch_select_keys(const Dims& dm, const float* qbar, const void* k_cache, const int32_t* kv_lens,
                              const int32_t* budgets, float* scores, int32_t* k_idx, int32_t* k_cnt, uint32_t* ws,
                              hipStream_t st, bool ws_is_zero) {
  const int n_keep = dm.n_ret < dm.C ? dm.n_ret : dm.C;
  if (!ws_is_zero) hipLaunchKernelGGL(sel_zero, dim3(64), dim3(256), 0, st, ws, select_keys_zero_words(dm));
  // provisional scores: the streaming kernel with the single bf16 term
  Dims prov = dm;
  prov.flags |= QUOKA_SCORE_QBAR_BF16;
  hipError_t e = launch_score_keys(prov, QUOKA_BF16, qbar, k_cache, kv_lens, scores, st);
  if (e != hipSuccess) return e;
  const dim3 grid(sel_tiles(dm.T_max), dm.n_kv, dm.b);
  hipLaunchKernelGGL(sel_hist, grid, dim3(kSelThreads), 0, st, dm, scores, kv_lens, budgets, ws);
  if (dm.d == 64) {
    launch_rescore<64>(dm, qbar, k_cache, kv_lens, budgets, scores, ws, n_keep, grid, st);
  } else {
    launch_rescore<128>(dm, qbar, k_cache, kv_lens, budgets, scores, ws, n_keep, grid, st);
  }
  hipLaunchKernelGGL(sel_band_select, dim3(dm.n_kv, dm.b), dim3(kSelHeadThreads), 0, st, dm, scores, kv_lens, budgets,
                     ws);
  hipLaunchKernelGGL(sel_emit, grid, dim3(kSelThreads), 0, st, dm, scores, kv_lens, budgets, ws, k_idx, k_cnt);
  return hipGetLastError();
}

}  // namespace quoka
