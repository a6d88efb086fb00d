// Tile arithmetic of the key scoring (Alg. 1: S = Qbar K^T, S-hat = max over the query axis; Sec. 3.2-3.3), shared
// by the streaming scoring kernel and by the exact re-scoring of the keys near the provisional cut: both must give
// the same float32 bits for the same key, so the split of Qbar, the order of the MFMA terms, the squared norm and
// the final division live here once.
//
// Operand plan (v_mfma_f32_32x32x16_bf16; a lane is (li = lane % 32, hf = lane / 32)): queries are the M side, keys
// the N side.  Lane (li, hf) holds, for k-step ks, dims ks*16 + 8*hf .. +8 of query row li (A) and of key li (B);
// the result block has key li in the lane and 16 query rows in its registers, so the max over queries is in-register
// plus one exchange between the half waves.
#pragma once
#include "common.hip.h"

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
  // two K tiles; three generations of squared norms and of per-query-block maxima (a tile's scores are finished
  // one step after its products, under the next tile's barrier)
  static constexpr size_t kLdsBytes = 2 * kTileBytes + 3 * kScTile * 4 + 3 * QB * kScTile * 4;
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// sum of squares of the 8 bf16 values of a 16-byte chunk (products of bf16 pairs are exact in float32)
__device__ __forceinline__ float sumsq_bf16x8(const u32x4& r) {
  // (the chunk is reinterpreted as a whole: casting single dwords of the vector to bf16 pairs is miscompiled)
  const bf16x8 v = __builtin_bit_cast(bf16x8, r);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bf16x2_t p = {v[2 * i], v[2 * i + 1]};
    s = __builtin_amdgcn_fdot2_f32_bf16(p, p, s, false);
  }
  return s;
}

// Squared norm of a key row whose CG 16-byte chunks sit in CG consecutive lanes (`r` is this lane's chunk).
template <int CG>
__device__ __forceinline__ float row_sumsq(const u32x4& r) {
  const float ss = sumsq_bf16x8(r);
  if constexpr (CG == 16) {
    return row16_sum(ss);   // a key row is exactly one 16-lane DPP row
  } else {
    return group_sum<CG>(ss);
  }
}

// Query operands of one wave: 32 rows of Qbar (rows qb*32 .. +32 of a head's [n_keep][D] float32 block) as bf16
// terms.  EXACT: hi + mid + lo add up to the float32 value exactly, so with bf16 keys every product is exact and only
// the float32 accumulation rounds.  Otherwise only hi (Qbar rounded to bf16) is formed.  Rows past n_keep repeat the
// last real query (the max is unchanged); `zero_pad` makes them zero instead (for the mean over queries).
template <int D, bool EXACT>
struct QueryTerms {
  bf16x8 hi[D / 16], mid[D / 16], lo[D / 16];
  __device__ __forceinline__ void load(const float* __restrict__ qhead, int n_keep, int qb, int li, int hf,
                                       bool zero_pad) {
    int r = qb * 32 + li;
    const bool pad_row = r >= n_keep;
    r = pad_row ? n_keep - 1 : r;
    const float* qrow = qhead + (size_t)r * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      const float4 x0 = *reinterpret_cast<const float4*>(qrow + ks * 16);
      const float4 x1 = *reinterpret_cast<const float4*>(qrow + ks * 16 + 4);
      float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
      if (zero_pad && pad_row) {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = 0.f;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const __bf16 h = (__bf16)x[e];
        hi[ks][e] = h;
        if constexpr (EXACT) {
          const float r1 = x[e] - (float)h;
          const __bf16 m = (__bf16)r1;
          const float r2 = r1 - (float)m;
          mid[ks][e] = m;
          lo[ks][e] = (__bf16)r2;
        }
      }
    }
  }
};

// Products of one wave over its share of a staged tile: keys kg*KPW .. +KPW of `tl` (row pitch LD) against the wave's
// 32 query rows; per key the max (or, mean_mode, the sum) over those rows goes to smax_g[qb*kScTile + key].  All
// three query terms go into one accumulator per key block (smallest term first inside every k-step), so there is
// nothing to add up afterwards; two key blocks are interleaved to keep the MFMA chains independent.
template <int D, int QB, bool EXACT>
__device__ __forceinline__ void tile_products(const uint16_t* __restrict__ tl, const QueryTerms<D, EXACT>& q, int qb,
                                              int kg, int li, int hf, bool mean_mode, float* __restrict__ smax_g) {
  using Cfg = ScoreCfg<D, QB>;
  constexpr int KS = Cfg::KS, LD = Cfg::LD, KPW = Cfg::KPW;
  constexpr int NKB = KPW / 32;
#pragma unroll
  for (int kb = 0; kb < NKB; kb += 2) {
    constexpr int kPair = NKB >= 2 ? 2 : 1;
    f32x16 c[kPair];
    const uint16_t* kp[kPair];
#pragma unroll
    for (int u = 0; u < kPair; ++u) {
      c[u] = f32x16{0};
      kp[u] = tl + (kg * KPW + (kb + u) * 32 + li) * LD + 8 * hf;
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 kop[kPair];
#pragma unroll
      for (int u = 0; u < kPair; ++u) kop[u] = *reinterpret_cast<const bf16x8*>(kp[u] + ks * 16);
      if constexpr (EXACT) {
#pragma unroll
        for (int u = 0; u < kPair; ++u) c[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q.lo[ks], kop[u], c[u], 0, 0, 0);
#pragma unroll
        for (int u = 0; u < kPair; ++u) c[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q.mid[ks], kop[u], c[u], 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < kPair; ++u) c[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q.hi[ks], kop[u], c[u], 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < kPair; ++u) {
      float m;
      if (mean_mode) {   // sum over this wave's 32 query rows (padding rows are zero)
        m = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) m += c[u][v];
        m += other_half(m);
      } else {
        m = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) m = fmaxf(m, c[u][v]);
        m = fmaxf(m, other_half(m));
      }
      if (hf == 0) smax_g[qb * kScTile + kg * KPW + (kb + u) * 32 + li] = m;
    }
  }
}

// Score of key `k` of a tile from the per-query-block maxima (sums) and the squared norm.
template <int QB>
__device__ __forceinline__ float tile_score(const float* __restrict__ sm, const float* __restrict__ ssq_g, int k,
                                            bool dot_mode, bool mean_mode, int n_keep) {
  float m = sm[k];
#pragma unroll
  for (int j = 1; j < QB; ++j) m = mean_mode ? m + sm[j * kScTile + k] : fmaxf(m, sm[j * kScTile + k]);
  if (mean_mode) m /= (float)n_keep;
  const float nrm = dot_mode ? 1.0f : fmaxf(sqrtf(ssq_g[k]), kNormEps);
  return m / nrm + 0.0f;
}

// Side job of a fused call: all blocks of the launch together clear `words` 32-bit words.
__device__ __forceinline__ void clear_words(uint32_t* __restrict__ p, uint32_t words) {
  if (p == nullptr) return;
  const uint32_t nblk = gridDim.x * gridDim.y * gridDim.z;
  const uint32_t blk = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  for (uint32_t i = blk * blockDim.x + threadIdx.x; i < words; i += nblk * blockDim.x) p[i] = 0u;
}

}  // namespace quoka
