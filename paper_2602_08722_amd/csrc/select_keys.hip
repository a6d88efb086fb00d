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
// Launch chain (no block ever waits for another block of its launch): provisional scoring with the histogram
// (score_stream.hip), band classification + exact re-scoring per 2048-key tile, one block per head that selects
// among the band candidates and lays out the tiles' output offsets, ordered emission per tile.
#include "common.hip.h"
#include "kernels.h"
#include "score_tile.hip.h"
#include "select_ws.hip.h"

namespace quoka {

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
// Band classification and exact re-scoring.  A block takes `tpb` consecutive 2048-key tiles of one head: it locates
// the band once from the finished histogram, then per tile classifies the keys and scores the band keys exactly.
template <int D, int QB>
__global__ __launch_bounds__(kSelThreads) void sel_band_rescore(Dims dm, const float* __restrict__ qbar,
                                                               const uint16_t* __restrict__ kc,
                                                               const int32_t* __restrict__ kv_lens,
                                                               const int32_t* __restrict__ budgets,
                                                               float* __restrict__ scores, uint32_t* __restrict__ ws,
                                                               int n_keep, int tpb) {
  using Cfg = ScoreCfg<D, QB>;
  constexpr int LD = Cfg::LD, CG = Cfg::CG, RPI = Cfg::RPI, NLD = Cfg::NLD;
  __shared__ __align__(16) uint16_t tile[kScTile * LD];
  __shared__ float ssq[kScTile];
  __shared__ float smax[QB * kScTile];
  __shared__ uint32_t band_loc[kSelTile];        // positions (relative to the tile) of the band keys, any order
  __shared__ uint32_t sh[kSelThreads + 2];
  __shared__ uint32_t bc[2];                     // cut bin, candidate slot base
  __shared__ uint32_t cnt2[2][2];                // per tile parity: band count, sure-in count

  const int kv = blockIdx.y, b = blockIdx.z;
  const SelCtx c = sel_ctx(dm, scores, kv_lens, budgets, ws, kv, b);
  const int tile_first = blockIdx.x * tpb;
  if (c.B == 0 || c.B >= c.T || tile_first * kSelTile >= c.T) return;   // block-uniform
  const int tile_end = min(tile_first + tpb, (c.T + kSelTile - 1) / kSelTile);
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qb = w % QB, kg = w / QB;
  const int li = lane & 31, hf = lane >> 5;
  if (tid < 4) (&cnt2[0][0])[tid] = 0u;

  // Everything the block needs from memory before it can classify is requested up front: the first tile's
  // provisional scores, the histogram, the error bound, and the query operands of the exact product.
  float p[kSelIPT];
  auto load_p = [&](int t0) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < kSelIPT; ++i) {
      const int t = t0 + tid + kSelThreads * i;   // coalesced rows
      p[i] = t < c.T ? c.sc[t] : 0.f;
    }
  };
  load_p(tile_first * kSelTile);
  constexpr uint32_t per = kSelBins / kSelThreads;
  const uint32_t top = kSelBins - tid * per;   // exclusive upper bin of this thread's run (thread 0: highest bins)
  uint32_t hv[per];
#pragma unroll
  for (uint32_t i = 0; i < per; i += 4) {
    const u32x4 v = *reinterpret_cast<const u32x4*>(c.w.hist + top - per + i);
    hv[i] = v[0]; hv[i + 1] = v[1]; hv[i + 2] = v[2]; hv[i + 3] = v[3];
  }
  const float d2 = __uint_as_float(c.w.meta[kMetaEps2]);
  QueryTerms<D, true> qt;
  qt.load(qbar + (size_t)c.head * n_keep * D, n_keep, qb, li, hf, false);

  // ---- the bin of the provisional cut: scanning from the top, where the running count reaches B ----
  {
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
  __syncthreads();
  // |p - s| <= ||delta|| (exact arithmetic; the scoring launch left the largest squared ||delta|| of the head) plus
  // the float32 accumulation and bin-edge slack of the two computed values
  const float eps = sqrtf(d2) * 1.001f + 4e-6f;
  const int m = (int)ceilf(2.0f * eps * (float)(kSelBins / 2)) + 1;
  const int cut_bin = (int)bc[0];
  const int bin_lo = max(cut_bin - m, 0), bin_hi = min(cut_bin + m, kSelBins - 1);
  if (blockIdx.x == 0 && tid == 0) {
    c.w.meta[kMetaBinLo] = (uint32_t)bin_lo;
    c.w.meta[kMetaBinHi] = (uint32_t)bin_hi;
  }
  const char* kbase = reinterpret_cast<const char*>(kc + b * dm.kvs[0] + kv * dm.kvs[1]);
  const uint32_t row_bytes = (uint32_t)dm.kvs[2] * 2u;
  const int cg = tid % CG, r0 = tid / CG;

  for (int tile_i = tile_first; tile_i < tile_end; ++tile_i) {
    const int t0 = tile_i * kSelTile;
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
        uint32_t* mw = c.w.mask + (size_t)tile_i * (kSelTile / 32) + (kSelThreads * i + 64 * w) / 32;
        mw[0] = (uint32_t)bal;
        mw[1] = (uint32_t)(bal >> 32);
      }
      uint32_t base = 0;
      if (lane == 0 && bal != 0) base = atomicAdd(&cnt2[tile_i & 1][0], (uint32_t)__popcll(bal));
      base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
      if (inb) band_loc[base + __popcll(bal & ((1ull << lane) - 1ull))] = (uint32_t)tl;
    }
    if (tile_i + 1 < tile_end) load_p(t0 + kSelTile);   // the next tile's scores travel during the re-scoring
    n_in = wave_incl_scan_u32(n_in);
    if (lane == 63 && n_in) atomicAdd(&cnt2[tile_i & 1][1], n_in);
    __syncthreads();
    const int n_band = (int)cnt2[tile_i & 1][0];
    if (tid == 0) {
      c.w.tile_in[tile_i] = cnt2[tile_i & 1][1];
      if (n_band > 0) bc[1] = atomicAdd(&c.w.meta[kMetaCand], (uint32_t)n_band);   // slots in the head's candidate list
      // the other parity's counters serve the next tile: their last readers passed the previous tile's second barrier
      cnt2[(tile_i + 1) & 1][0] = 0u;
      cnt2[(tile_i + 1) & 1][1] = 0u;
    }
    __syncthreads();
    const uint32_t slot0 = bc[1];

    // ---- exact scores of the band keys, 128 at a time, by the tile arithmetic of the streaming kernel ----
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
      __syncthreads();   // the tile, norms and maxima are overwritten by the next batch (and band_loc by the next tile)
    }
  }
}

// ---------------------------------------------------------------------------------------------
// One block per head: the exact cut among the band candidates, then the output offset of every tile.
// Radix select (descending) over keys that are read again from memory in every pass (the candidate list of a head is
// a few tens of KiB and stays in cache; there is no bound on its length, so registers cannot hold it in general).
struct HeadSelectLds {
  RadixSelectLds rs;
  uint32_t wsum[kSelHeadThreads / 64 + 1];
};

__device__ __forceinline__ void stream_radix_select_desc(const uint32_t* __restrict__ keys, uint32_t n, uint32_t need,
                                                         RadixSelectLds& L, uint32_t* cut_key, uint32_t* need_eq) {
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
  const u32x4 hv = *reinterpret_cast<const u32x4*>(c.w.hist + 4 * tid);
  const uint32_t bin_hi = c.w.meta[kMetaBinHi];
  const uint32_t n_c = c.w.meta[kMetaCand];
  uint32_t n_in = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) n_in += (uint32_t)(4 * tid + i) > bin_hi ? hv[i] : 0u;
  uint32_t tot_in;
  block_excl_scan<kSelHeadThreads>(n_in, L.wsum, &tot_in);
  const uint32_t need = (uint32_t)c.B - tot_in;   // >= 1: fewer than B keys lie above the cut bin, let alone the band
  for (int i = tid; i < nt; i += kSelHeadThreads) cnt[i] = 0u;
  __syncthreads();
  // (the candidates are read again from memory in every pass: holding them in registers, 16 per thread, was
  // measured slower -- 13.5 against 11.2 us at 4000 candidates per head)
  uint32_t tau, need_eq;
  stream_radix_select_desc(c.w.cand_key, n_c, need, L.rs, &tau, &need_eq);
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
                           const int32_t* budgets, float* scores, uint32_t* ws, int n_keep, hipStream_t st) {
  // one round of two blocks per compute unit: fewer, fatter blocks amortise the histogram scan and the query operands
  // (mixed-length batch of 8 x 8 heads: 37 us with 512 blocks, 41 with 1024, 49 with 2048)
  const int heads = dm.b * dm.n_kv, nt = sel_tiles(dm.T_max);
  const int per_head = (512 + heads - 1) / heads;
  const int tpb = (nt + per_head - 1) / per_head;
  const dim3 grid((nt + tpb - 1) / tpb, dm.n_kv, dm.b);
  const int qblocks = (n_keep + 31) / 32;
  const uint16_t* k = static_cast<const uint16_t*>(kc);
  if (qblocks <= 1) {
    hipLaunchKernelGGL((sel_band_rescore<D, 1>), grid, dim3(kSelThreads), 0, st, dm, qbar, k, kv_lens, budgets, scores,
                       ws, n_keep, tpb);
  } else if (qblocks == 2) {
    hipLaunchKernelGGL((sel_band_rescore<D, 2>), grid, dim3(kSelThreads), 0, st, dm, qbar, k, kv_lens, budgets, scores,
                       ws, n_keep, tpb);
  } else {
    hipLaunchKernelGGL((sel_band_rescore<D, 4>), grid, dim3(kSelThreads), 0, st, dm, qbar, k, kv_lens, budgets, scores,
                       ws, n_keep, tpb);
  }
}

hipError_t launch_select_keys(const Dims& dm, const float* qbar, const void* k_cache, const int32_t* kv_lens,
                              const int32_t* budgets, float* scores, int32_t* k_idx, int32_t* k_cnt, uint32_t* ws,
                              hipStream_t st, bool ws_is_zero) {
  const int n_keep = dm.n_ret < dm.C ? dm.n_ret : dm.C;
  if (!ws_is_zero) hipLaunchKernelGGL(sel_zero, dim3(64), dim3(256), 0, st, ws, select_keys_zero_words(dm));
  // provisional scores and their histogram in one streaming launch
  hipError_t e = launch_score_stream(dm, qbar, k_cache, kv_lens, scores, ws, st);
  if (e != hipSuccess) return e;
  const dim3 grid(sel_tiles(dm.T_max), dm.n_kv, dm.b);
  if (dm.d == 64) {
    launch_rescore<64>(dm, qbar, k_cache, kv_lens, budgets, scores, ws, n_keep, st);
  } else {
    launch_rescore<128>(dm, qbar, k_cache, kv_lens, budgets, scores, ws, n_keep, st);
  }
  hipLaunchKernelGGL(sel_band_select, dim3(dm.n_kv, dm.b), dim3(kSelHeadThreads), 0, st, dm, scores, kv_lens, budgets,
                     ws);
  hipLaunchKernelGGL(sel_emit, grid, dim3(kSelThreads), 0, st, dm, scores, kv_lens, budgets, ws, k_idx, k_cnt);
  return hipGetLastError();
}

}  // namespace quoka
