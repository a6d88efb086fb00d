// Chunk attention on bf16 MFMA (Alg. 2 attention step; Eq. 2-3): flash-style online softmax over
// [gathered cache rows | chunk rows], causal inside the chunk.  One kernel serves the sparse path
// (rows gathered through k_idx while the tile is staged into LDS -- the reduced cache of Eq. 3 is
// never materialised) and the dense baseline of Eq. 2 (rows 0..kv_len).
//
// Work split: a wave owns a row block: 32 query rows of one q-head.  Row blocks of a KV head are numbered
// (token tile, head-in-group), and a block's waves take half of their row blocks from the front of that list
// and half from the back, so every block (and, with two waves per SIMD, every SIMD) gets the same mix of
// short and long causal ranges.  All waves of a block share every staged K/V tile.
//
// MFMA operand plan (v_mfma_f32_32x32x16_bf16; a lane is (li = lane % 32, hf = lane / 32)):
//   S^T[key, row] = K[key, :] . Q[row, :]      A = K tile rows from LDS, B = Q held in registers.
//     Result layout: lane li = query row, 16 registers = keys 8*(v/4) + 4*hf + v%4 of a 32-key block.
//     Row max / row sum are therefore in-lane plus one exchange between the two half waves.
//   O^T[dim, row] += V[key, dim] . P[row, key]  B = P: exactly the registers S^T left in the lane
//     (the contraction index may be permuted freely, so no transpose or shuffle is needed),
//     A = V^T, fetched from the row-major LDS tile with the transposing LDS read (ds_read_b64_tr_b16):
//     in every group of 16 lanes, lane s supplies the address of 4 consecutive dims of one key, and
//     lane L receives dim (L % 4) of the four lanes L/4, L/4 + 4, L/4 + 8, L/4 + 12.  With lane s
//     pointing at key row0 + s/4, dims dim0 + 4*(s%4), lane L ends up with dim dim0 + L of keys
//     row0 .. row0+3: a quarter of an MFMA A operand, with no register shuffling.
//     Accumulator block c, register v of lane li holds O[row li, dim 32*c + 8*(v/4) + 4*hf + v%4].
#include "common.hip.h"
#include "kernels.h"

namespace quoka {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef s16x4 __attribute__((address_space(3))) * tr_ptr;   // LDS address of one lane's 8 bytes of a transposing read

constexpr int kBN = 64;   // keys per staged tile

// NW = waves per wave set (4 or 8); a block holds NSETS wave sets.
template <int D, int NW>
struct AttnCfg {
  static constexpr int kThreads = 64 * NW;
  static constexpr int KS = D / 16;              // k-steps of the QK^T product
  static constexpr int LD = D + 8;               // padded LDS row of the K tile (elements)
  static constexpr int LDV = D + 32;             // V tile: rows 64 bytes apart modulo 256, so the 8 rows x 64 bytes
                                                 // one transposing read touches fall on distinct banks per half wave
  static constexpr int CG = D / 8;               // 16-byte chunks per row
  static constexpr int RPI = kThreads / CG;    // rows per block-wide load
  static constexpr int NLD = kBN / RPI;          // loads per thread per tile (per tensor)
  static constexpr int DB = D / 32;              // dim blocks of the PV product
  static constexpr size_t kKTileBytes = (size_t)kBN * LD * 2;
  static constexpr size_t kStageBytes = kKTileBytes + (size_t)kBN * LDV * 2;   // one K tile and one V tile
  static constexpr size_t kLdsBytes = 2 * kStageBytes;                          // double buffered
};

// NSETS = 1: one set of NW waves.  NSETS = 2 (NW = 4): waves 4-7 take the same 4 row blocks as waves 0-3 but every
// other KV tile (own LDS buffers, same barriers), and the two partial results are merged through LDS at the end.
// This puts two waves on every SIMD when the grid alone cannot.  The second set's waves are rotated by two
// against the first's, so each SIMD hosts one front (short) and one back (long) row block.
template <int D, int NW, int NSETS>
__global__ __launch_bounds__(64 * NW * NSETS, 2) void attn_bf16(Dims dm, AttnArgs a) {
  using Cfg = AttnCfg<D, NW>;
  constexpr int KS = Cfg::KS, LD = Cfg::LD, LDV = Cfg::LDV, CG = Cfg::CG, RPI = Cfg::RPI, NLD = Cfg::NLD, DB = Cfg::DB;
  constexpr int kThreads = Cfg::kThreads, HW = NW / 2;
  extern __shared__ __align__(16) unsigned char smem[];

  const int kv = blockIdx.x, b = blockIdx.z;   // KV head fastest: one head's blocks share an XCD's L2
  const int tid = threadIdx.x % kThreads, lane = tid & 63;                    // position inside the wave set
  // wave-uniform values are pinned to scalar registers so that everything derived from them (tile kind, base
  // pointers, branches) stays scalar too
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int set = NSETS == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x / kThreads);
  unsigned char* const smem_set = smem + (size_t)set * Cfg::kLdsBytes;
  const int li = lane & 31, hf = lane >> 5;
  const int C = dm.C, g = dm.g;
  const int ntt = (C + 31) / 32;
  const int nrb = g * ntt;                       // row blocks of this KV head
  const int half = (nrb + 1) / 2;                // row blocks [0, half) are "front", [half, nrb) "back"
  const int slot = NSETS == 1 ? w : (w + HW * set) % NW;   // slots [0, HW) front, [HW, NW) back
  const bool back = slot >= HW;
  const int kf = blockIdx.y * HW + slot % HW;
  const int x = back ? nrb - 1 - kf : kf;
  const bool wave_on = back ? (x >= half) : (x < half);
  const int xj = wave_on ? x % g : 0;
  const int tok0 = wave_on ? (x / g) * 32 : 0;
  const int h = kv * g + xj;
  const int xb_hi = nrb - 1 - (int)blockIdx.y * HW;                                     // the block's last row block
  const int x_hi = xb_hi >= half ? xb_hi : min((int)blockIdx.y * HW + HW - 1, half - 1);
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
  // K and V of this (batch, KV head), as byte pointers: every row is addressed as base + 32-bit byte offset
  // (the host checks that a head's rows span less than 4 GiB), which keeps the per-tile address arithmetic
  // to one multiply-add per staged row.
  const char* kcache = reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.k_cache) + b * dm.kvs[0] + kv * dm.kvs[1]);
  const char* vcache = reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.v_cache) + b * dm.kvs[0] + kv * dm.kvs[1]);
  const char* kchunk = reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.k_chunk) + b * dm.cks[0] + kv * dm.cks[1]);
  const char* vchunk = reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.v_chunk) + b * dm.cks[0] + kv * dm.cks[1]);
  const char* kidx = sparse ? reinterpret_cast<const char*>(a.k_idx + (size_t)(b * dm.n_kv + kv) * dm.B_max) : nullptr;
  const uint32_t cache_row_bytes = (uint32_t)dm.kvs[2] * 2u, chunk_row_bytes = (uint32_t)dm.cks[2] * 2u;

  // Q operand: row tok0 + li, dims ks*16 + 8*hf .. +8
  bf16x8 qreg[KS];
  {
    const int tok = min(tok0 + li, C - 1);
    const uint16_t* qrow = qg + b * dm.qs[0] + h * dm.qs[1] + (size_t)tok * dm.qs[2] + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
  }

  const int cg = tid % CG, r0 = tid / CG;
  uint32_t rows[NLD];   // source rows of the tile to be issued next
  u32x4 RK[NLD], RV[NLD];

  // Source rows of a tile are resolved one tile ahead of the loads that use them, so the dependent
  // index -> row fetch of the gather never sits on the critical path: the fetched indices are first touched
  // when the next tile's loads are issued, after the wait the LDS stores need anyway.  (Written as macros, not
  // lambdas: the staging registers must stay in VGPRs.)
#define QUOKA_RESOLVE(IT)                                                                          \
  do {                                                                                             \
    const int it_ = (IT);                                                                          \
    if (it_ < n_tiles) {                                                                           \
      const bool cache_ = it_ < n_ct;                                                              \
      const int base_ = cache_ ? it_ * kBN : (it_ - n_ct) * kBN;                                   \
      const int last_ = cache_ ? n_cache - 1 : C - 1;                                              \
      if (cache_ && sparse) {                                                                      \
        _Pragma("unroll") for (int i = 0; i < NLD; ++i) {                                          \
          const uint32_t n_ = (uint32_t)min(base_ + r0 + RPI * i, last_); /* tail slots repeat a real row */ \
          rows[i] = *reinterpret_cast<const uint32_t*>(kidx + n_ * 4u);                            \
        }                                                                                          \
      } else {                                                                                     \
        _Pragma("unroll") for (int i = 0; i < NLD; ++i)                                            \
          rows[i] = (uint32_t)min(base_ + r0 + RPI * i, last_);                                    \
      }                                                                                            \
    }                                                                                              \
  } while (0)
#define QUOKA_ISSUE(IT)                                                                            \
  do {                                                                                             \
    const bool cache_ = (IT) < n_ct;                                                               \
    const char* kb_ = cache_ ? kcache : kchunk;                                                    \
    const char* vb_ = cache_ ? vcache : vchunk;                                                    \
    const uint32_t rb_ = cache_ ? cache_row_bytes : chunk_row_bytes;                               \
    _Pragma("unroll") for (int i = 0; i < NLD; ++i) {                                              \
      const uint32_t off_ = rows[i] * rb_ + (uint32_t)cg * 16u;                                    \
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
    uint16_t* kt = reinterpret_cast<uint16_t*>(smem_set + (size_t)(j & 1) * Cfg::kStageBytes);
    uint16_t* vt = kt + kBN * LD;
    if (has_tile) {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int rl = r0 + RPI * i;
        *reinterpret_cast<u32x4*>(kt + rl * LD + cg * 8) = RK[i];
        *reinterpret_cast<u32x4*>(vt + rl * LDV + cg * 8) = RV[i];
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
    __builtin_amdgcn_s_setprio(2);   // the wave feeding the matrix core goes first; its SIMD mate fills the gaps
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int v = 0; v < 16; ++v) s[nb][v] = __builtin_amdgcn_exp2f(fmaf(s[nb][v], sl2, -m_use));
    // ---- O^T += V^T P^T -----------------------------------------------------------------------
    // lane's corner of every transposing read: key 4*hf + (lane%16)/4, dims 16*((lane/16)%2) + 4*(lane%4)
    const tr_ptr vtr = (tr_ptr)(vt + (4 * hf + ((lane & 15) >> 2)) * LDV + 16 * ((lane >> 4) & 1) + 4 * (lane & 3));
    float psum = 0.f;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        // k-slot e of this lane is key 16t + 8*(e/4) + 4*hf + e%4 of block nb
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[e] = (__bf16)s[nb][8 * t + e];
        // row sum of the probabilities as the matrix core sees them (rounded to bf16)
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const bf16x2 pp = {pb[e], pb[e + 1]};
          psum = __builtin_amdgcn_fdot2_f32_bf16(pp, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, psum, false);
        }
#pragma unroll
        for (int c = 0; c < DB; ++c) {
          const int e0 = (nb * 32 + 16 * t) * LDV + c * 32;   // elements past the lane's corner
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(vtr + e0 / 4);
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(vtr + (e0 + 8 * LDV) / 4);
          const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pb, o[c], 0, 0, 0);
        }
      }
    }
    l_run += psum;
    __builtin_amdgcn_s_setprio(0);
  }

  // ---- merge of the two wave sets (NSETS == 2): set 1 hands (m, l, O) to set 0 through LDS ------------------------
  if constexpr (NSETS == 2) {
    constexpr int REC = 2 + DB * 16;
    float* mg = reinterpret_cast<float*>(smem) + (size_t)(slot * 64 + lane) * REC;   // both sets' waves of a slot share rows
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
    for (int c = 0; c < DB; ++c)
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {   // registers 4*v4 .. 4*v4+3 are four consecutive dims
        uint2 pk;
        pk.x = f32_to_bf16_bits(o[c][4 * v4] * inv) | (f32_to_bf16_bits(o[c][4 * v4 + 1] * inv) << 16);
        pk.y = f32_to_bf16_bits(o[c][4 * v4 + 2] * inv) | (f32_to_bf16_bits(o[c][4 * v4 + 3] * inv) << 16);
        *reinterpret_cast<uint2*>(orow + 32 * c + 8 * v4 + 4 * hf) = pk;
      }
    if (a.lse != nullptr && hf == 0) {
      a.lse[(size_t)(b * dm.n_q + h) * C + tok] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
    }
  }
}

#undef QUOKA_RESOLVE
#undef QUOKA_ISSUE

template <int D, int NW, int NSETS>
static hipError_t launch_dn(const Dims& dm, const AttnArgs& a, hipStream_t st) {
  using Cfg = AttnCfg<D, NW>;
  constexpr size_t lds = NSETS * Cfg::kLdsBytes;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16<D, NW, NSETS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int nrb = dm.g * ((dm.C + 31) / 32);
  const int half = (nrb + 1) / 2;
  dim3 grid(dm.n_kv, (half + NW / 2 - 1) / (NW / 2), dm.b);
  hipLaunchKernelGGL((attn_bf16<D, NW, NSETS>), grid, dim3(Cfg::kThreads * NSETS), lds, st, dm, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const Dims& dm, const AttnArgs& a, hipStream_t st) {
  constexpr int kComputeUnits = 256;   // MI355X
  const int nrb = dm.g * ((dm.C + 31) / 32);
  const long long blocks4 = (long long)dm.n_kv * (((nrb + 1) / 2 + 1) / 2) * dm.b;
  // fewer than two 4-wave blocks per compute unit: use 8-wave blocks that split the KV tiles between two wave sets
  if (blocks4 >= 2 * kComputeUnits) return launch_dn<D, 4, 1>(dm, a, st);
  return launch_dn<D, 4, 2>(dm, a, st);
}

hipError_t launch_attn_bf16(const Dims& dm, const AttnArgs& a, hipStream_t st) {
  return dm.d == 64 ? launch_d<64>(dm, a, st) : launch_d<128>(dm, a, st);
}

}  // namespace quoka
