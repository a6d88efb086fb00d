// Top-B key selection per (sequence, KV head) (Alg. 1: I = topk(S-hat, B_SA); Eq. 3).
//
// Exact radix select on order-preserving uint32 images of the float scores, then an ordered
// compaction so that indices come out in ascending position and equal scores go to the lower
// position.  Integer work only: the result is deterministic and independent of the launch shape.
//
//   T_max <= kSmallMax : one 1024-thread block per head, keys held in registers, one launch.
//   larger             : several blocks per head.  Three histogram passes (11 + 11 + 10 bits, global
//                        integer atomics) find the cut key; a count pass and an emit pass produce
//                        the ordered index list.  Each launch derives the newest step of the cut
//                        from the histogram the previous launch completed (and leaves it in the
//                        workspace for the later ones), so no kernel waits on another block.
#include "common.hip.h"
#include "kernels.h"

namespace quoka {

constexpr int kSmallMax = 32768;   // beyond this one compute unit is slower than the multi-block path
constexpr int kSmallThreads = 1024;
constexpr int kLgThreads = 256;
constexpr int kLgTile = 2048;          // scores per block in the multi-block path
constexpr int kBins = 2048;            // bins per histogram pass (11 bits; last pass uses 1024)

__device__ __forceinline__ int radix_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ uint32_t radix_bins(int pass) { return pass == 2 ? 1024u : 2048u; }

// ---------------------------------------------------------------------------------------------
// Single-block path.  Wave w owns scores [w*64*IPT, (w+1)*64*IPT); its register j of lane l is score
// w*64*IPT + 64*j + l, so every load is a coalesced 256-byte row and position order inside a wave is (j, lane).
// The cut key comes from the block-wide radix select; the ordered compaction needs no scan over threads: per
// register, two wave ballots give every lane the number of earlier taken positions of its wave, and the 16 wave
// totals are combined through LDS.

template <int IPT>
__global__ __launch_bounds__(kSmallThreads) void topk_small(Dims dm, const float* __restrict__ scores,
                                                           const int32_t* __restrict__ kv_lens,
                                                           const int32_t* __restrict__ budgets,
                                                           int32_t* __restrict__ k_idx, int32_t* __restrict__ k_cnt) {
  constexpr int NW = kSmallThreads / 64;
  __shared__ RadixSelectLds rs;
  __shared__ uint32_t wgt[NW], weq[NW];
  const int kv = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const float* sc = scores + (size_t)(b * dm.n_kv + kv) * dm.T_max;
  const int lo = w * 64 * IPT + lane;   // position of register 0; register j is 64*j further
  // The scores are requested before the cache length is known (the row has T_max entries; those past the length
  // are discarded below), so the two fetches overlap instead of queueing behind each other.
  float raw[IPT];
#pragma unroll
  for (int j = 0; j < IPT; ++j) raw[j] = lo + 64 * j < dm.T_max ? sc[lo + 64 * j] : 0.f;
  const int T = max(0, min(kv_lens[b], dm.T_max));
  const int B = max(0, min(min(budgets[b], T), dm.B_max));
  int32_t* out = k_idx + (size_t)(b * dm.n_kv + kv) * dm.B_max;
  if (tid == 0) k_cnt[b * dm.n_kv + kv] = B;
  if (B == 0) return;
  if (B >= T) {
    for (int i = tid; i < T; i += kSmallThreads) out[i] = i;
    return;
  }
  uint32_t key[IPT];
  uint32_t valid = 0u;
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    const bool in = lo + 64 * j < T;
    key[j] = in ? max(okey(raw[j]), 1u) : 0u;   // real keys are never 0, so the padding can neither exceed nor equal a cut key
    valid |= (in ? 1u : 0u) << j;
  }
  uint32_t tau, need_eq;
  block_radix_select<IPT, true>(key, valid, (uint32_t)B, rs, &tau, &need_eq);   // descending: the B largest
  // wave totals of (key > tau) and (key == tau): per-lane counts (both in one register: at most 32 each), one scan
  uint32_t cnt = 0;
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    cnt += (key[j] > tau ? 0x10000u : 0u) + (key[j] == tau ? 1u : 0u);
  }
  cnt = wave_incl_scan_u32(cnt);
  if (lane == 63) {
    wgt[w] = cnt >> 16;
    weq[w] = cnt & 0xFFFFu;
  }
  __syncthreads();
  // taken candidates at earlier positions (earlier waves): greater than the cut / equal to it
  uint32_t n_gt = wave_incl_scan_u32(lane < w ? wgt[lane] : 0u);
  uint32_t n_eq = wave_incl_scan_u32(lane < w ? weq[lane] : 0u);
  n_gt = (uint32_t)__builtin_amdgcn_readlane((int)n_gt, 63);
  n_eq = (uint32_t)__builtin_amdgcn_readlane((int)n_eq, 63);
  const unsigned long long below = (1ull << lane) - 1ull;
  // (an opaque copy of the cut: otherwise the comparison masks of the counting loop above are kept alive for this
  // loop, 2 x IPT scalar register pairs that spill)
  uint32_t tau_e = tau;
  asm volatile("" : "+v"(tau_e));
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    const int t = lo + 64 * j;
    const bool gt = key[j] > tau_e, eq = key[j] == tau_e;
    const unsigned long long m_gt = __builtin_amdgcn_ballot_w64(gt), m_eq = __builtin_amdgcn_ballot_w64(eq);
    const uint32_t gt_before = n_gt + __popcll(m_gt & below), eq_before = n_eq + __popcll(m_eq & below);
    if (gt || (eq && eq_before < need_eq)) {   // equal scores go to the lower positions
      const uint32_t pos = gt_before + min(eq_before, need_eq);
      if (pos < (uint32_t)B) out[pos] = t;     // guard: a malformed score array cannot push writes past the budget
    }
    n_gt += __popcll(m_gt);
    n_eq += __popcll(m_eq);
    __builtin_amdgcn_sched_barrier(0);   // keep one register's ballots live at a time (32 pairs would spill SGPRs)
  }
}

// ---------------------------------------------------------------------------------------------
// Multi-block path.  Workspace per head: hist[3][kBins] then tile counts [n_tiles][2].
struct Cut {
  uint32_t prefix;  // decided high bits of the cut key
  uint32_t mask;    // which bits are decided
  uint32_t need;    // rank of the cut inside the remaining candidates (1-based, descending)
};

// Whole block: locate the bin (scanning from the top) where the running count reaches `need`.
// Returns (bin, need reduced by the counts above that bin).  `sh` is LDS scratch [kLgThreads + 2].
__device__ __forceinline__ void find_bin(const uint32_t* __restrict__ hist, uint32_t nbins, uint32_t need,
                                         uint32_t* sh, uint32_t* bin_out, uint32_t* need_out) {
  // thread t owns bins [nbins - (t+1)*per, nbins - t*per): thread 0 has the highest bins.
  const uint32_t per = nbins / kLgThreads;
  const uint32_t top = nbins - threadIdx.x * per;   // exclusive upper bin
  uint32_t mine = 0;
  for (uint32_t i = 1; i <= per; ++i) mine += hist[top - i];
  uint32_t tot;
  const uint32_t above = block_excl_scan<kLgThreads>(mine, sh, &tot);   // count in all higher-bin threads
  __syncthreads();
  if (above < need && need <= above + mine) {   // exactly one thread (need <= total is guaranteed)
    uint32_t rem = need - above;
    uint32_t i = 1;
    for (; i <= per; ++i) {
      const uint32_t c = hist[top - i];
      if (rem <= c) break;
      rem -= c;
    }
    sh[kLgThreads] = top - i;
    sh[kLgThreads + 1] = rem;
  }
  __syncthreads();
  *bin_out = sh[kLgThreads];
  *need_out = sh[kLgThreads + 1];
  __syncthreads();
}

// The cut after `npass` finished histogram passes.  Every pass adds one step (a bin and the rank left inside it).  A
// kernel works out only the newest step, from the histogram the previous launch completed; the steps before it are
// read back from `cuts` (two words per step), where block 0 of the launch that first derived them has left them
// (`newest_stored`: a previous launch has already derived the newest step too).
__device__ __forceinline__ Cut derive_cut(const uint32_t* __restrict__ hist, uint32_t* __restrict__ cuts, int npass,
                                          bool newest_stored, uint32_t B, uint32_t* sh) {
  Cut c{0u, 0u, B};
  for (int p = 0; p < npass; ++p) {
    uint32_t bin, need;
    if (p + 1 < npass || newest_stored) {
      bin = cuts[2 * p];
      need = cuts[2 * p + 1];
    } else {
      find_bin(hist + p * kBins, radix_bins(p), c.need, sh, &bin, &need);
      if (blockIdx.x == 0 && threadIdx.x == 0) {
        cuts[2 * p] = bin;
        cuts[2 * p + 1] = need;
      }
    }
    const int sft = radix_shift(p);
    c.prefix |= bin << sft;
    c.mask |= (radix_bins(p) - 1u) << sft;
    c.need = need;
  }
  return c;
}

__global__ void topk_zero(uint32_t* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

constexpr int kCutWords = 8;   // three (bin, rank) steps, padded
struct LgCtx {
  int T, B;
  const float* sc;
  uint32_t* hist;
  uint32_t* cuts;
  uint32_t* tcnt;
};

__device__ __forceinline__ LgCtx lg_ctx(const Dims& dm, const float* scores, const int32_t* kv_lens,
                                        const int32_t* budgets, uint32_t* ws, int n_tiles) {
  const int kv = blockIdx.y, b = blockIdx.z;
  LgCtx c;
  c.T = max(0, min(kv_lens[b], dm.T_max));
  c.B = max(0, min(min(budgets[b], c.T), dm.B_max));
  const size_t head = (size_t)(b * dm.n_kv + kv);
  c.sc = scores + head * dm.T_max;
  const size_t per_head = 3 * (size_t)kBins + kCutWords + 2 * (size_t)n_tiles;
  c.hist = ws + head * per_head;
  c.cuts = c.hist + 3 * kBins;
  c.tcnt = c.cuts + kCutWords;
  return c;
}

template <int PASS>
__global__ __launch_bounds__(kLgThreads) void topk_hist(Dims dm, const float* __restrict__ scores,
                                                       const int32_t* __restrict__ kv_lens,
                                                       const int32_t* __restrict__ budgets, uint32_t* __restrict__ ws,
                                                       int n_tiles) {
  __shared__ uint32_t lh[kBins];
  __shared__ uint32_t sh[kLgThreads + 2];
  const LgCtx c = lg_ctx(dm, scores, kv_lens, budgets, ws, n_tiles);
  const int t0 = blockIdx.x * kLgTile;
  if (c.B == 0 || c.B >= c.T || t0 >= c.T) return;   // block-uniform
  const Cut cut = derive_cut(c.hist, c.cuts, PASS, false, (uint32_t)c.B, sh);
  for (int i = threadIdx.x; i < kBins; i += kLgThreads) lh[i] = 0;
  __syncthreads();
  const int sft = radix_shift(PASS);
  const uint32_t bm = radix_bins(PASS) - 1u;
  const int t1 = min(t0 + kLgTile, c.T);
  for (int i = t0 + threadIdx.x; i < t1; i += kLgThreads) {
    const uint32_t k = okey(c.sc[i]);
    if ((k & cut.mask) == cut.prefix) atomicAdd(&lh[(k >> sft) & bm], 1u);
  }
  __syncthreads();
  uint32_t* gh = c.hist + PASS * kBins;
  for (int i = threadIdx.x; i < kBins; i += kLgThreads) {
    const uint32_t v = lh[i];
    if (v) atomicAdd(&gh[i], v);
  }
}

// EMIT == false: per-tile counts of (key > cut, key == cut).  EMIT == true: ordered output.
template <bool EMIT>
__global__ __launch_bounds__(kLgThreads) void topk_finish(Dims dm, const float* __restrict__ scores,
                                                         const int32_t* __restrict__ kv_lens,
                                                         const int32_t* __restrict__ budgets,
                                                         uint32_t* __restrict__ ws, int n_tiles,
                                                         int32_t* __restrict__ k_idx, int32_t* __restrict__ k_cnt) {
  __shared__ uint32_t sh[kLgThreads + 2];
  const LgCtx c = lg_ctx(dm, scores, kv_lens, budgets, ws, n_tiles);
  const int kv = blockIdx.y, b = blockIdx.z;
  const int t0 = blockIdx.x * kLgTile;
  int32_t* out = k_idx + (size_t)(b * dm.n_kv + kv) * dm.B_max;
  if (EMIT && blockIdx.x == 0 && threadIdx.x == 0) k_cnt[b * dm.n_kv + kv] = c.B;
  if (c.B == 0 || t0 >= c.T) return;
  const int t1 = min(t0 + kLgTile, c.T);
  if (c.B >= c.T) {
    if (EMIT)
      for (int i = t0 + threadIdx.x; i < t1; i += kLgThreads) out[i] = i;
    return;
  }
  const Cut cut = derive_cut(c.hist, c.cuts, 3, EMIT, (uint32_t)c.B, sh);   // the count pass leaves the last step for the emit pass
  const uint32_t tau = cut.prefix, need_eq = cut.need;
  // thread t owns kLgTile / kLgThreads consecutive scores
  constexpr int IPT = kLgTile / kLgThreads;
  const int lo = t0 + threadIdx.x * IPT;
  uint32_t kreg[IPT];
  uint32_t cnt = 0;   // keys above the cut in the high half, keys equal to it in the low half (at most 2048 per tile)
#pragma unroll
  for (int i = 0; i < IPT; ++i) {
    const int t = lo + i;
    const uint32_t k = t < t1 ? okey(c.sc[t]) : 0u;   // 0 is below every real key image except okey(-NaN); never > tau
    kreg[i] = k;
    cnt += ((t < t1) && (k > tau) ? 0x10000u : 0u) + ((t < t1) && (k == tau) ? 1u : 0u);
  }
  uint32_t tot;
  const uint32_t before = block_excl_scan<kLgThreads>(cnt, sh, &tot);
  if (!EMIT) {
    if (threadIdx.x == 0) {
      c.tcnt[2 * blockIdx.x] = tot >> 16;
      c.tcnt[2 * blockIdx.x + 1] = tot & 0xFFFFu;
    }
    return;
  }
  const uint32_t p_gt = before >> 16;
  uint32_t p_eq = before & 0xFFFFu;
  // counts of all earlier tiles (fixed order; at most a few hundred tiles): per-thread partial sums, one wave scan
  // each, the four wave totals through LDS
  uint32_t e_gt = 0, e_eq = 0;
  for (int i = threadIdx.x; i < (int)blockIdx.x; i += kLgThreads) {
    e_gt += c.tcnt[2 * i];
    e_eq += c.tcnt[2 * i + 1];
  }
  e_gt = wave_incl_scan_u32(e_gt);
  e_eq = wave_incl_scan_u32(e_eq);
  __syncthreads();   // sh is free again
  if ((threadIdx.x & 63) == 63) {
    sh[threadIdx.x >> 6] = e_gt;
    sh[kLgThreads / 64 + (threadIdx.x >> 6)] = e_eq;
  }
  __syncthreads();
  uint32_t before_gt = 0, before_eq = 0;
#pragma unroll
  for (int i = 0; i < kLgThreads / 64; ++i) {
    before_gt += sh[i];
    before_eq += sh[kLgThreads / 64 + i];
  }
  p_eq += before_eq;
  uint32_t pos = before_gt + p_gt + min(p_eq, need_eq);
#pragma unroll
  for (int i = 0; i < IPT; ++i) {
    const int t = lo + i;
    if (t < t1) {
      const uint32_t k = kreg[i];
      bool take = k > tau;
      if (k == tau) {
        take = p_eq < need_eq;
        ++p_eq;
      }
      if (take) {
        if (pos < (uint32_t)c.B) out[pos] = t;
        ++pos;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
static inline int lg_tiles(const Dims& dm) { return (dm.T_max + kLgTile - 1) / kLgTile; }

size_t topk_ws_words(const Dims& dm) {
  if (dm.T_max <= kSmallMax) return 0;
  return (size_t)dm.b * dm.n_kv * (3 * (size_t)kBins + kCutWords + 2 * (size_t)lg_tiles(dm));
}

hipError_t launch_topk_keys(const Dims& dm, const float* scores, const int32_t* kv_lens, const int32_t* budgets,
                            int32_t* k_idx, int32_t* k_cnt, uint32_t* ws, hipStream_t st, bool ws_is_zero) {
  if (dm.T_max <= kSmallMax) {
    const dim3 grid(dm.n_kv, dm.b), block(kSmallThreads);
    const int ipt = (dm.T_max + kSmallThreads - 1) / kSmallThreads;
    if (ipt <= 1) {
      hipLaunchKernelGGL((topk_small<1>), grid, block, 0, st, dm, scores, kv_lens, budgets, k_idx, k_cnt);
    } else if (ipt <= 2) {
      hipLaunchKernelGGL((topk_small<2>), grid, block, 0, st, dm, scores, kv_lens, budgets, k_idx, k_cnt);
    } else if (ipt <= 4) {
      hipLaunchKernelGGL((topk_small<4>), grid, block, 0, st, dm, scores, kv_lens, budgets, k_idx, k_cnt);
    } else if (ipt <= 8) {
      hipLaunchKernelGGL((topk_small<8>), grid, block, 0, st, dm, scores, kv_lens, budgets, k_idx, k_cnt);
    } else if (ipt <= 16) {
      hipLaunchKernelGGL((topk_small<16>), grid, block, 0, st, dm, scores, kv_lens, budgets, k_idx, k_cnt);
    } else {
      hipLaunchKernelGGL((topk_small<32>), grid, block, 0, st, dm, scores, kv_lens, budgets, k_idx, k_cnt);
    }
    return hipGetLastError();
  }
  const int n_tiles = lg_tiles(dm);
  const size_t words = topk_ws_words(dm);
  if (!ws_is_zero) hipLaunchKernelGGL(topk_zero, dim3(256), dim3(256), 0, st, ws, words);
  dim3 grid(n_tiles, dm.n_kv, dm.b);
  hipLaunchKernelGGL((topk_hist<0>), grid, dim3(kLgThreads), 0, st, dm, scores, kv_lens, budgets, ws, n_tiles);
  hipLaunchKernelGGL((topk_hist<1>), grid, dim3(kLgThreads), 0, st, dm, scores, kv_lens, budgets, ws, n_tiles);
  hipLaunchKernelGGL((topk_hist<2>), grid, dim3(kLgThreads), 0, st, dm, scores, kv_lens, budgets, ws, n_tiles);
  hipLaunchKernelGGL((topk_finish<false>), grid, dim3(kLgThreads), 0, st, dm, scores, kv_lens, budgets, ws, n_tiles,
                     k_idx, k_cnt);
  hipLaunchKernelGGL((topk_finish<true>), grid, dim3(kLgThreads), 0, st, dm, scores, kv_lens, budgets, ws, n_tiles,
                     k_idx, k_cnt);
  return hipGetLastError();
}

}  // namespace quoka
