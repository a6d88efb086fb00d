// Constants, score binning and workspace layout shared by the kernels of the scoring + top-B stage for long caches.
#pragma once
#include "common.hip.h"

namespace quoka {

constexpr int kSelBins = 4096;        // equal bins over [-1, 1]
constexpr int kSelTile = 2048;        // keys per block in the per-tile kernels
constexpr int kSelThreads = 256;
constexpr int kSelIPT = kSelTile / kSelThreads;
constexpr int kSelMeta = 16;          // per-head words: candidate count, band limits, exact cut
constexpr int kSelHeadThreads = 1024;
constexpr int kSelMaxTiles = (1 << 24) / kSelTile;   // the interface limits a cache to 2^24 - 1 positions

enum { kMetaCand = 0, kMetaBinLo = 1, kMetaBinHi = 2, kMetaTau = 3, kMetaNeedEq = 4, kMetaEps2 = 5 };

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

}  // namespace quoka
