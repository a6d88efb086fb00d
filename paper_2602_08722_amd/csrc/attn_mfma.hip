// Chunk attention on bf16 MFMA (Alg. 2 attention step; Eq. 2-3): flash-style online softmax over
// [gathered cache rows | chunk rows], causal inside the chunk.  One kernel serves the sparse path
// (rows gathered through k_idx while the tile is staged into LDS -- the reduced cache of Eq. 3 is
// never materialised) and the dense baseline of Eq. 2 (rows 0..kv_len).
//
// Work split: a wave owns 32 query rows of one q-head; the four waves of a block take four
// consecutive (token tile, head-in-group) row blocks of one KV head, so with a group of 4 the block's
// waves are the 4 q-heads that share every staged K/V tile.
//
// MFMA operand plan (v_mfma_f32_32x32x16_bf16; a lane is (li = lane % 32, hf = lane / 32)):
//   S^T[key, row] = K[key, :] . Q[row, :]      A = K tile rows from LDS, B = Q held in registers.
//     Result layout: lane li = query row, 16 registers = keys 8*(v/4) + 4*hf + v%4 of a 32-key block.
//     Row max / row sum are therefore in-lane plus one exchange between the two half waves.
//   O^T[dim, row] += V[key, dim] . P[row, key]  B = P: exactly the registers S^T left in the lane
//     (the contraction index may be permuted freely, so no transpose or shuffle is needed),
//     A = V read from the row-major LDS tile as DB consecutive dims per lane: lane li takes dims
//     DB*li .. DB*li+DB-1 of 8 keys and feeds one element to each of the DB dim-blocks.
//     Accumulator block c, register v of lane li holds O[row li, dim DB*(8*(v/4)+4*hf+v%4) + c].
#include "common.hip.h"
#include "kernels.h"

namespace quoka {

constexpr int kAtThreads = 256;
constexpr int kBN = 64;   // keys per staged tile

template <int D>
struct AttnCfg {
  static constexpr int KS = D / 16;              // k-steps of the QK^T product
  static constexpr int LD = D + 8;               // padded LDS row (elements)
  static constexpr int CG = D / 8;               // 16-byte chunks per row
  static constexpr int RPI = kAtThreads / CG;    // rows per block-wide load
  static constexpr int NLD = kBN / RPI;          // loads per thread per tile (per tensor)
  static constexpr int DB = D / 32;              // dim blocks of the PV product
  static constexpr size_t kTileBytes = (size_t)kBN * LD * 2;
  static constexpr size_t kLdsBytes = 4 * kTileBytes;  // K and V, double buffered
};

// NSETS = 1: a block is 4 waves.  NSETS = 2: a block is 8 waves; waves 4-7 take the same 4 row blocks as waves 0-3
// but every other KV tile (own LDS buffers, same barriers), and the two partial results are merged through LDS at
// the end.  This puts two waves on every SIMD when the grid alone cannot (one row block per SIMD), so one wave's
// softmax overlaps the other's MFMAs.
template <int D, int NSETS>
__global__ __launch_bounds__(kAtThreads * NSETS, 2) void attn_bf16(Dims dm, AttnArgs a) {
  using Cfg = AttnCfg<D>;
  constexpr int KS = Cfg::KS, LD = Cfg::LD, CG = Cfg::CG, RPI = Cfg::RPI, NLD = Cfg::NLD, DB = Cfg::DB;
  extern __shared__ __align__(16) unsigned char smem[];

  const int kv = blockIdx.x, b = blockIdx.z;   // KV head fastest: one head's blocks share an XCD's L2
  const int tid = threadIdx.x % kAtThreads, lane = tid & 63, w = tid >> 6;   // position inside the wave set
  const int set = threadIdx.x / kAtThreads;
  unsigned char* const smem_set = smem + (size_t)set * Cfg::kLdsBytes;
  const int li = lane & 31, hf = lane >> 5;
  const int C = dm.C, g = dm.g;
  const int ntt = (C + 31) / 32;
  const int nrb = g * ntt;                       // row blocks of this KV head
  const int x = blockIdx.y * 4 + w;
  const bool wave_on = x < nrb;
  const int xj = wave_on ? x % g : 0;
  const int tok0 = wave_on ? (x / g) * 32 : 0;
  const int h = kv * g + xj;
  const int x_hi = min((int)blockIdx.y * 4 + 3, nrb - 1);
  const int c_end_blk = min((x_hi / g) * 32 + 32, C);   // chunk keys any wave of this block can see

  const bool sparse = a.k_idx != nullptr;
  int n_cache;
  if (sparse) {
    n_cache = min(a.n_cache[b * dm.n_kv + kv], dm.B_max);
  } else {
    n_cache = min(a.n_cache[b], dm.T_max);
  }
  n_cache = max(n_cache, 0);
  const int n_ct = (n_cache + kBN - 1) / kBN;
  const int n_tiles = n_ct + (c_end_blk + kBN - 1) / kBN;

  const uint16_t* qg = static_cast<const uint16_t*>(a.q);
  const uint16_t* kcache = static_cast<const uint16_t*>(a.k_cache) + b * dm.kvs[0] + kv * dm.kvs[1];
  const uint16_t* vcache = static_cast<const uint16_t*>(a.v_cache) + b * dm.kvs[0] + kv * dm.kvs[1];
  const uint16_t* kchunk = static_cast<const uint16_t*>(a.k_chunk) + b * dm.cks[0] + kv * dm.cks[1];
  const uint16_t* vchunk = static_cast<const uint16_t*>(a.v_chunk) + b * dm.cks[0] + kv * dm.cks[1];
  const int32_t* kidx = sparse ? a.k_idx + (size_t)(b * dm.n_kv + kv) * dm.B_max : nullptr;

  // Q operand: row tok0 + li, dims ks*16 + 8*hf .. +8
  bf16x8 qreg[KS];
  {
    const int tok = min(tok0 + li, C - 1);
    const uint16_t* qrow = qg + b * dm.qs[0] + h * dm.qs[1] + (size_t)tok * dm.qs[2] + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
  }

  const int cg = tid % CG, r0 = tid / CG;
  int rows[NLD];       // resolved source rows of the tile to be issued next
  u32x4 RK[NLD], RV[NLD];

  // Source rows of a tile are resolved one tile ahead of the loads that use them, so the dependent
  // index -> row fetch of the gather never sits on the critical path.  (Written as macros, not lambdas:
  // the staging registers must stay in VGPRs.)
#define QUOKA_RESOLVE(IT)                                                                          \
  do {                                                                                             \
    const int it_ = (IT);                                                                          \
    if (it_ < n_tiles) {                                                                           \
      const bool cache_ = it_ < n_ct;                                                              \
      const int base_ = cache_ ? it_ * kBN : (it_ - n_ct) * kBN;                                   \
      const int last_ = cache_ ? n_cache - 1 : C - 1;                                              \
      _Pragma("unroll") for (int i = 0; i < NLD; ++i) {                                            \
        const int n_ = min(base_ + r0 + RPI * i, last_); /* tail slots repeat a real row */        \
        rows[i] = (cache_ && sparse) ? kidx[n_] : n_;                                              \
      }                                                                                            \
    }                                                                                              \
  } while (0)
#define QUOKA_ISSUE(IT)                                                                            \
  do {                                                                                             \
    const bool cache_ = (IT) < n_ct;                                                               \
    const uint16_t* kb_ = cache_ ? kcache : kchunk;                                                \
    const uint16_t* vb_ = cache_ ? vcache : vchunk;                                                \
    const long long st_ = cache_ ? dm.kvs[2] : dm.cks[2];                                          \
    _Pragma("unroll") for (int i = 0; i < NLD; ++i) {                                              \
      const size_t off_ = (size_t)rows[i] * st_ + cg * 8;                                          \
      RK[i] = *reinterpret_cast<const u32x4*>(kb_ + off_);                                         \
      RV[i] = *reinterpret_cast<const u32x4*>(vb_ + off_);                                         \
    }                                                                                              \
  } while (0)

  QUOKA_RESOLVE(set);
  if (set < n_tiles) QUOKA_ISSUE(set);
  QUOKA_RESOLVE(set + NSETS);

  f32x16 o[DB];
#pragma unroll
  for (int c = 0; c < DB; ++c)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[c][v] = 0.f;
  float m_run = -INFINITY;   // running row max, in the scaled log2 domain
  float l_run = 0.f;         // this half wave's share of the running row sum
  const float sl2 = 1.4426950408889634f / sqrtf((float)D);
  const int tok = tok0 + li;

  const int n_steps = (n_tiles + NSETS - 1) / NSETS;
  for (int j = 0; j < n_steps; ++j) {
    const int it = j * NSETS + set;       // this wave set's tile of the step
    const bool has_tile = it < n_tiles;
    uint16_t* kt = reinterpret_cast<uint16_t*>(smem_set + (size_t)(j & 1) * 2 * Cfg::kTileBytes);
    uint16_t* vt = kt + kBN * LD;
    if (has_tile) {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int rl = r0 + RPI * i;
        *reinterpret_cast<u32x4*>(kt + rl * LD + cg * 8) = RK[i];
        *reinterpret_cast<u32x4*>(vt + rl * LD + cg * 8) = RV[i];
      }
    }
    __syncthreads();   // tile `it` visible; every wave is past its reads of the other buffer's previous use
    if (it + NSETS < n_tiles) {
      QUOKA_ISSUE(it + NSETS);
      QUOKA_RESOLVE(it + 2 * NSETS);
    }
    if (!has_tile) continue;

    const bool is_chunk = it >= n_ct;
    const int base = is_chunk ? (it - n_ct) * kBN : it * kBN;   // first key of the tile in its own numbering
    if (!wave_on || (is_chunk && base > tok0 + 31)) continue;   // tile entirely in this wave's future

    // ---- S^T = K Q^T --------------------------------------------------------------------------
    f32x16 s[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) s[nb][v] = 0.f;
      const uint16_t* kp = kt + (nb * 32 + li) * LD + 8 * hf;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 kop = *reinterpret_cast<const bf16x8*>(kp + ks * 16);
        s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop, qreg[ks], s[nb], 0, 0, 0);
      }
    }
    // ---- mask ---------------------------------------------------------------------------------
    const int limit = is_chunk ? (tok - base + 1) : (n_cache - base);   // keys kk < limit are visible
    if (limit < kBN) {   // lane-varying for chunk tiles; only comparisons, no cross-lane traffic inside
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int kk = nb * 32 + 8 * (v / 4) + 4 * hf + (v % 4);
          if (kk >= limit) s[nb][v] = -INFINITY;
        }
    }
    // ---- online softmax -----------------------------------------------------------------------
    // The reference point m_run only moves when the tile maximum exceeds it by more than 2^kLazy:
    // exp2(s - m_run) then stays below 2^kLazy, and rescaling the accumulators becomes rare.
    float mx = -INFINITY;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[nb][v]);
    mx = fmaxf(mx, other_half(mx)) * sl2;
    constexpr float kLazy = 8.0f;
    if (__builtin_amdgcn_ballot_w64(mx > m_run + kLazy) != 0) {   // wave-uniform branch
      const float m_new = (mx > m_run + kLazy) ? mx : m_run;       // -inf + 8 = -inf: the first visible tile lands here
      const float m_fin = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_fin);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int c = 0; c < DB; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[c][v] *= alpha;
    }
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
    float psum = 0.f;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[nb][v], sl2, -m_use));
        s[nb][v] = p;
        psum += p;
      }
    l_run += psum;
    // ---- O^T += V^T P^T -----------------------------------------------------------------------
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[e] = (__bf16)s[nb][8 * t + e];
        // the 8 keys behind this lane's k-slots: 16t + 8*(e/4) + 4*hf + e%4 of block nb
        uint32_t vr[8][DB / 2];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int kk = nb * 32 + 16 * t + 8 * (e / 4) + 4 * hf + (e % 4);
          const uint16_t* vp = vt + kk * LD + DB * li;
          if constexpr (DB == 4) {
            const u32x2 r = *reinterpret_cast<const u32x2*>(vp);
            vr[e][0] = r[0];
            vr[e][1] = r[1];
          } else {
            vr[e][0] = *reinterpret_cast<const uint32_t*>(vp);
          }
        }
#pragma unroll
        for (int c = 0; c < DB; ++c) {
          // dim block c takes 16-bit element c of every read: byte-permute pairs of keys into one dword
          const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
          u32x4 packed;
#pragma unroll
          for (int p2 = 0; p2 < 4; ++p2)
            packed[p2] = __builtin_amdgcn_perm(vr[2 * p2 + 1][c / 2], vr[2 * p2][c / 2], sel);
          const bf16x8 vop = __builtin_bit_cast(bf16x8, packed);
          o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, pb, o[c], 0, 0, 0);
        }
      }
    }
  }

  // ---- merge of the two wave sets (NSETS == 2): set 1 hands (m, l, O) to set 0 through LDS ------------------------
  if constexpr (NSETS == 2) {
    constexpr int REC = 2 + DB * 16;
    float* mg = reinterpret_cast<float*>(smem) + (size_t)(w * 64 + lane) * REC;
    __syncthreads();   // all tiles consumed: the tile buffers may be reused
    if (set == 1) {
      mg[0] = m_run;
      mg[1] = l_run;
#pragma unroll
      for (int c = 0; c < DB; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) mg[2 + c * 16 + v] = o[c][v];
    }
    __syncthreads();
    if (set == 1) return;
    const float m1 = mg[0], l1 = mg[1];
    const float m_new = fmaxf(m_run, m1);
    const float m_fin = (m_new == -INFINITY) ? 0.f : m_new;
    const float a0 = __builtin_amdgcn_exp2f(m_run - m_fin), a1 = __builtin_amdgcn_exp2f(m1 - m_fin);
    m_run = m_new;
    l_run = a0 * l_run + a1 * l1;
#pragma unroll
    for (int c = 0; c < DB; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[c][v] = a0 * o[c][v] + a1 * mg[2 + c * 16 + v];
  }

  // ---- epilogue -------------------------------------------------------------------------------
  const float l_tot = l_run + other_half(l_run);
  if (wave_on && tok < C) {
    const float inv = 1.0f / l_tot;
    uint16_t* orow = static_cast<uint16_t*>(a.out) + b * dm.os[0] + h * dm.os[1] + (size_t)tok * dm.os[2];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int iv = 8 * (v / 4) + 4 * hf + (v % 4);
      if constexpr (DB == 4) {
        uint2 pk;
        pk.x = f32_to_bf16_bits(o[0][v] * inv) | (f32_to_bf16_bits(o[1][v] * inv) << 16);
        pk.y = f32_to_bf16_bits(o[2][v] * inv) | (f32_to_bf16_bits(o[3][v] * inv) << 16);
        *reinterpret_cast<uint2*>(orow + 4 * iv) = pk;
      } else {
        const uint32_t pk = f32_to_bf16_bits(o[0][v] * inv) | (f32_to_bf16_bits(o[1][v] * inv) << 16);
        *reinterpret_cast<uint32_t*>(orow + 2 * iv) = pk;
      }
    }
    if (a.lse != nullptr && hf == 0) {
      a.lse[(size_t)(b * dm.n_q + h) * C + tok] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
    }
  }
}

#undef QUOKA_RESOLVE
#undef QUOKA_ISSUE

template <int D, int NSETS>
static hipError_t launch_dn(const Dims& dm, const AttnArgs& a, int n_blocks_y, hipStream_t st) {
  using Cfg = AttnCfg<D>;
  constexpr size_t lds = NSETS * Cfg::kLdsBytes;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16<D, NSETS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  dim3 grid(dm.n_kv, n_blocks_y, dm.b);
  hipLaunchKernelGGL((attn_bf16<D, NSETS>), grid, dim3(kAtThreads * NSETS), lds, st, dm, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const Dims& dm, const AttnArgs& a, hipStream_t st) {
  constexpr int kComputeUnits = 256;   // MI355X
  const int nrb = dm.g * ((dm.C + 31) / 32);
  const int ny = (nrb + 3) / 4;
  const long long blocks = (long long)dm.n_kv * ny * dm.b;
  // fewer than two 4-wave blocks per compute unit: use 8-wave blocks that split the KV tiles between two wave sets
  if (blocks < 2 * kComputeUnits) return launch_dn<D, 2>(dm, a, ny, st);
  return launch_dn<D, 1>(dm, a, ny, st);
}

hipError_t launch_attn_bf16(const Dims& dm, const AttnArgs& a, hipStream_t st) {
  return dm.d == 64 ? launch_d<64>(dm, a, st) : launch_d<128>(dm, a, st);
}

}  // namespace quoka
