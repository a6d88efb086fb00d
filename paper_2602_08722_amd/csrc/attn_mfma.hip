// Chunk attention on bf16 MFMA (Alg. 2 attention step; Eq. 2-3): flash-style online softmax over
// [gathered cache rows | chunk rows], causal inside the chunk.  One kernel serves the sparse path
// (rows gathered through k_idx while the tile is staged into LDS -- the reduced cache of Eq. 3 is
// never materialised) and the dense baseline of Eq. 2 (rows 0..kv_len).
//
// Work split: a wave owns a row block: 32 query rows of one q-head.  Row blocks of a KV head are numbered
// (token tile, head-in-group).  In a launch of one round a block takes half of its row blocks from the front of that
// list and half from the back, so every block (and every SIMD, which hosts one wave of each kind) gets the same mix of
// short and long causal ranges; in a launch of several rounds a block takes neighbouring row blocks and the blocks
// with the longest ranges come first.  A block is two sets of four waves that share every staged K/V tile.
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
//
// Schedule: the two wave sets run half a step apart.  While one set forms S = K Q^T of a tile (matrix core only)
// the other runs softmax and P V (exponentials interleaved with MFMAs), then they swap.  A SIMD hosts one wave of
// each set, so its matrix core always has one wave that only feeds it and one whose vector work fills the gaps.
// Two barriers per step keep the halves aligned and protect the double-buffered LDS stages.
#include "common.hip.h"
#include "kernels.h"

namespace quoka {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef s16x4 __attribute__((address_space(3))) * tr_ptr;   // LDS address of one lane's 8 bytes of a transposing read

constexpr int kComputeUnits = 256;   // MI355X
constexpr int kSetThreads = 256;   // four waves
constexpr int kSub = 64;           // keys a wave set consumes per step

// SPLIT = false: the sets own different row blocks (8 per block) and both consume every 64-key tile.
// SPLIT = true:  both sets own the same 4 row blocks; a staged tile has 128 keys, set s consumes keys 64*s..64*s+63,
//                and the two partial results are merged through LDS at the end.  Used when 8 row blocks per block
//                would leave compute units without a block.
// Index of the sequence whose length has descending rank `rank` among lens[0], lens[stride], ... (nb <= 64 of them; ties
// keep batch order).  Every wave works it out for itself: one load, nb lane reads, a ballot.
__device__ __forceinline__ int seq_of_rank(const int32_t* __restrict__ lens, int stride, int nb, int rank) {
  const int lane = threadIdx.x & 63;
  const int mine = lane < nb ? lens[lane * stride] : -1;
  int r = 0;
  for (int j = 0; j < nb; ++j) {
    const int other = __builtin_amdgcn_readlane(mine, j);
    r += (other > mine) || (other == mine && j < lane);
  }
  const unsigned long long hit = __builtin_amdgcn_ballot_w64(lane < nb && r == rank);
  return hit ? (int)__builtin_ctzll(hit) : rank;
}

template <int D, bool SPLIT>
struct AttnCfg {
  static constexpr int KT = SPLIT ? 2 * kSub : kSub;  // keys per staged tile
  static constexpr int KS = D / 16;                   // k-steps of the QK^T product
  static constexpr int LD = D + 8;                    // padded LDS row of the K tile (elements)
  static constexpr int LDV = D + 32;                  // V tile: rows 64 bytes apart modulo 256, so the 8 rows x 64 bytes
                                                      // one transposing read touches fall on distinct banks per half wave
  static constexpr int CG = D / 8;                    // 16-byte chunks per row
  static constexpr int RPI = kSetThreads / CG;        // rows per set-wide load
  static constexpr int NLD = KT / RPI;                // loads per thread per tile (set 0 loads K, set 1 loads V)
  static constexpr int DB = D / 32;                   // dim blocks of the PV product
  static constexpr int HW = SPLIT ? 2 : 4;            // front (= back) row blocks per block
  static constexpr size_t kKTileBytes = (size_t)KT * LD * 2;
  static constexpr size_t kStageBytes = kKTileBytes + (size_t)KT * LDV * 2;   // one K tile and one V tile
  static constexpr size_t kLdsBytes = 2 * kStageBytes;                          // double buffered
};

// XS (QUOKA_ATTN_SCALE_F32): the softmax scale is applied to the float32 products, one fused multiply-add per score
// together with the subtraction of the reference point.  Otherwise the factor log2(e)/sqrt(d) is folded into the bf16 Q
// operand once and the accumulator of K Q^T starts from minus the reference point, so that the matrix core hands back
// what the exponential takes and no vector instruction is spent on either -- 4-9 % faster, at the price of rounding Q a
// second time: an error of the logits of relative size 2^-9, which shows in the output once the logits are several
// times those of unit-variance inputs (0.03 absolute at four times, 0.06 at eight).
template <int D, bool SPLIT, bool XS>
__global__ __launch_bounds__(2 * kSetThreads, 2) void attn_bf16(Dims dm, AttnArgs a) {
  using Cfg = AttnCfg<D, SPLIT>;
  constexpr int KT = Cfg::KT, KS = Cfg::KS, LD = Cfg::LD, LDV = Cfg::LDV, CG = Cfg::CG, RPI = Cfg::RPI, NLD = Cfg::NLD,
                DB = Cfg::DB, HW = Cfg::HW;
  extern __shared__ __align__(16) unsigned char smem[];

  const int kv = blockIdx.x;   // KV head fastest: one head's blocks share an XCD's L2
  const bool sparse = a.k_idx != nullptr;
  // Blocks are dispatched in grid order and a block runs as long as its sequence's key list, so in a ragged batch the
  // sequences are taken longest first (grid slice z works on the sequence of rank z by attended cache length);
  // otherwise a long sequence that happens to come last starts when most of the chip has already drained.
  int b = blockIdx.z;
  if (dm.b > 1 && dm.b <= kWave)
    b = seq_of_rank(sparse ? a.n_cache + kv : a.n_cache, sparse ? dm.n_kv : 1, dm.b, blockIdx.z);
  const int tid = threadIdx.x % kSetThreads, lane = tid & 63;                 // position inside the wave set
  // wave-uniform values are pinned to scalar registers so that everything derived from them (tile kind, base
  // pointers, branches) stays scalar too
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int set = __builtin_amdgcn_readfirstlane(threadIdx.x / kSetThreads);
  const int li = lane & 31, hf = lane >> 5;
  const int C = dm.C, g = dm.g;
  const int ntt = (C + 31) / 32;
  const int nrb = g * ntt;                       // row blocks of this KV head
  const int half = (nrb + 1) / 2;                // row blocks [0, half) are "front", [half, nrb) "back"
  // SPLIT: slots 0,1 front, 2,3 back, and set 1's waves are rotated by two so that each SIMD hosts a front and a back
  // row block.  Otherwise set 0 is front, set 1 back.
  const int slot = SPLIT ? (w + 2 * set) % 4 : w + 4 * set;
  const bool back = SPLIT ? slot >= 2 : set == 1;
  const int kf = blockIdx.y * HW + slot % HW;
  // Row blocks of a block.  Paired (a launch of one round): half from the front of the list, half from the back, so all
  // blocks take equally long.  Adjacent (a launch of several rounds): 2*HW neighbours with nearly the same causal range,
  // so no wave idles while others still have chunk keys to go, and the blocks with the longest ranges come first
  // in the grid: the compute units that finish the short blocks early pick up more of what is left.
  const bool adjacent = a.adjacent != 0;
  const int x = adjacent ? nrb - 1 - ((int)blockIdx.y * 2 * HW + slot) : (back ? nrb - 1 - kf : kf);
  const bool wave_on = adjacent ? x >= 0 : (back ? (x >= half) : (x < half));
  const int xj = wave_on ? x % g : 0;
  const int tok0 = wave_on ? (x / g) * 32 : 0;
  const int h = kv * g + xj;
  const int xb_hi = nrb - 1 - (int)blockIdx.y * HW;                                     // the block's last row block
  const int x_hi = adjacent ? nrb - 1 - (int)blockIdx.y * 2 * HW
                            : (xb_hi >= half ? xb_hi : min((int)blockIdx.y * HW + HW - 1, half - 1));
  const int c_end_blk = min((x_hi / g) * 32 + 32, C);   // chunk keys any wave of this block can see
  const int sub = SPLIT ? set * kSub : 0;               // first key of this set's share of a staged tile

  int n_cache;
  if (sparse) {
    n_cache = min(a.n_cache[b * dm.n_kv + kv], dm.B_max);
  } else {
    n_cache = min(a.n_cache[b], dm.T_max);
  }
  n_cache = max(n_cache, 0);
  // Tile order: the chunk's own tiles first, then the cache tiles.  The online softmax does not care, and the first
  // chunk tile needs no index look-up and no cache length, so its loads leave right at kernel start.
  const int n_cht = (c_end_blk + KT - 1) / KT;
  const int n_ct = (n_cache + KT - 1) / KT;
  const int n_tiles = n_cht + n_ct;

  const uint16_t* qg = static_cast<const uint16_t*>(a.q);
  // The tensor this set stages (set 0: K, set 1: V) for this (batch, KV head), as byte pointers: every row is
  // addressed as base + 32-bit byte offset (the host checks that a head's rows span less than 4 GiB).
  const void* cache_t = set == 0 ? a.k_cache : a.v_cache;
  const void* chunk_t = set == 0 ? a.k_chunk : a.v_chunk;
  const char* cache_base = reinterpret_cast<const char*>(static_cast<const uint16_t*>(cache_t) + b * dm.kvs[0] + kv * dm.kvs[1]);
  const char* chunk_base = reinterpret_cast<const char*>(static_cast<const uint16_t*>(chunk_t) + b * dm.cks[0] + kv * dm.cks[1]);
  const char* kidx = sparse ? reinterpret_cast<const char*>(a.k_idx + (size_t)(b * dm.n_kv + kv) * dm.B_max) : nullptr;
  const uint32_t cache_row_bytes = (uint32_t)dm.kvs[2] * 2u, chunk_row_bytes = (uint32_t)dm.cks[2] * 2u;
  const int ld_mine = set == 0 ? LD : LDV;                              // LDS row pitch of the tensor this set stages
  const size_t stage_off_mine = set == 0 ? 0 : Cfg::kKTileBytes;      // its place inside a stage

  // Q operand: row tok0 + li, dims ks*16 + 8*hf .. +8
  bf16x8 qreg[KS];
  {
    const int tokq = min(tok0 + li, C - 1);
    const uint16_t* qrow = qg + b * dm.qs[0] + h * dm.qs[1] + (size_t)tokq * dm.qs[2] + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
  }
  // the softmax scale and the change to base 2
  const float qscale = 1.4426950408889634f / sqrtf((float)D);
  if constexpr (!XS) {   // into Q once, so K Q^T arrives in the exponent's own units
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) qreg[ks][e] = (__bf16)((float)qreg[ks][e] * qscale);
  }

  const int cg = tid % CG, r0 = tid / CG;
  const uint32_t idx_max = (uint32_t)max(dm.T_max - 1, 0);
  uint32_t rows[NLD];   // source rows of the tile to be issued next
  u32x4 R[NLD];         // staging registers of the tile in flight

  // Source rows of a tile are resolved one tile ahead of the loads that use them, so the dependent
  // index -> row fetch of the gather never sits on the critical path: the fetched indices are first touched
  // when the next tile's loads are issued, after the wait the LDS stores need anyway.  (Written as macros, not
  // lambdas: the staging registers must stay in VGPRs.)
#define QUOKA_RESOLVE(IT)                                                                          \
  do {                                                                                             \
    const int it_ = (IT);                                                                          \
    if (it_ < n_tiles) {                                                                           \
      const bool cache_ = it_ >= n_cht;                                                            \
      const int base_ = cache_ ? (it_ - n_cht) * KT : it_ * KT;                                    \
      const int last_ = cache_ ? n_cache - 1 : C - 1;                                              \
      if (cache_ && sparse) {                                                                      \
        _Pragma("unroll") for (int i = 0; i < NLD; ++i) {                                          \
          const uint32_t n_ = (uint32_t)min(base_ + r0 + RPI * i, last_); /* tail slots repeat a real row */ \
          rows[i] = *reinterpret_cast<const uint32_t*>(kidx + n_ * 4u); /* clamped where it is used */ \
        }                                                                                          \
      } else {                                                                                     \
        _Pragma("unroll") for (int i = 0; i < NLD; ++i)                                            \
          rows[i] = (uint32_t)min(base_ + r0 + RPI * i, last_);                                    \
      }                                                                                            \
    }                                                                                              \
  } while (0)
#define QUOKA_ISSUE(IT)                                                                            \
  do {                                                                                             \
    const bool cache_ = (IT) >= n_cht;                                                             \
    const char* tb_ = cache_ ? cache_base : chunk_base;                                            \
    const uint32_t rb_ = cache_ ? cache_row_bytes : chunk_row_bytes;                               \
    /* Cache rows are clamped to the cache extent: a malformed list (negative or too large) cannot leave the tensor. \
       The clamp sits here, not where the index is fetched: there it would make every wave wait for the fetch it \
       has just issued. */                                                                          \
    const uint32_t row_max_ = cache_ ? idx_max : 0xffffffffu;                                      \
    _Pragma("unroll") for (int i = 0; i < NLD; ++i)                                                \
      R[i] = *reinterpret_cast<const u32x4*>(tb_ + (min(rows[i], row_max_) * rb_ + (uint32_t)cg * 16u)); \
  } while (0)

  // tile 0 is the first chunk tile (the chunk is never empty): no index, no cache length
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    rows[i] = (uint32_t)min(r0 + RPI * i, C - 1);
    R[i] = *reinterpret_cast<const u32x4*>(chunk_base + (rows[i] * chunk_row_bytes + (uint32_t)cg * 16u));
  }
  QUOKA_RESOLVE(1);

  f32x16 o[DB];
#pragma unroll
  for (int c = 0; c < DB; ++c)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[c][v] = 0.f;
  float m_run = -INFINITY;   // running row max, in the scaled log2 domain
  float l_run = 0.f;         // this half wave's share of the running row sum
  // What the accumulator of K Q^T starts from.  !XS: -m_use in every entry, so the matrix core hands back s - m_use
  // and the exponential needs no subtraction of its own; rewritten only when the reference point moves.  XS: zero.
  f32x16 cinit;
#pragma unroll
  for (int v = 0; v < 16; ++v) cinit[v] = 0.f;
  const int tok = tok0 + li;
  f32x16 s[2];               // S^T of the tile between its two halves

  // first key (in the tile's own numbering: cache slot or chunk position) of this set's share of tile t
  auto share_base = [&](int t) { return (t >= n_cht ? t - n_cht : t) * KT + sub; };
  // whether this wave has anything visible in its share of tile t
  auto computes = [&](int t) {
    if (!wave_on || t < 0 || t >= n_tiles) return false;
    const int base = share_base(t);
    return t < n_cht ? base <= tok0 + 31 : base < n_cache;
  };

  // ---- first half of a tile: S^T = K Q^T ---------------------------------------------------------
  auto qk = [&](int t) __attribute__((always_inline)) {
    const uint16_t* kt = reinterpret_cast<const uint16_t*>(smem + (size_t)(t & 1) * Cfg::kStageBytes);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const uint16_t* kp = kt + (sub + nb * 32 + li) * LD + 8 * hf;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 kop = *reinterpret_cast<const bf16x8*>(kp + ks * 16);
        s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop, qreg[ks], ks == 0 ? cinit : s[nb], 0, 0, 0);
      }
    }
  };

  // ---- second half: mask, online softmax, O^T += V^T P^T ---------------------------------------
  auto softmax_pv = [&](int t) __attribute__((always_inline)) {
    const bool is_chunk = t < n_cht;
    const int base = share_base(t);
    const uint16_t* vt =
        reinterpret_cast<const uint16_t*>(smem + (size_t)(t & 1) * Cfg::kStageBytes + Cfg::kKTileBytes) + sub * LDV;
    const int limit = is_chunk ? (tok - base + 1) : (n_cache - base);   // keys kk < limit are visible
    if (limit < kSub) {   // lane-varying for chunk tiles; only comparisons, no cross-lane traffic inside
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int kk = nb * 32 + 8 * (v / 4) + 4 * hf + (v % 4);
          if (kk >= limit) s[nb][v] = -INFINITY;
        }
    }
    // The reference point m_run only moves when the tile maximum exceeds it by more than 2^kLazy:
    // exp2(s - m_run) then stays below 2^kLazy, and rescaling the accumulators becomes rare.
    float mx = -INFINITY;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[nb][v]);
    mx = fmaxf(mx, other_half(mx));
    constexpr float kLazy = 8.0f;
    if constexpr (XS) {
      mx *= qscale;   // the row's largest score of this tile, scaled log2 domain (the products themselves are raw)
      const bool moves = m_run == -INFINITY ? mx > -INFINITY : mx > m_run + kLazy;
      if (__builtin_amdgcn_ballot_w64(moves) != 0) {   // wave-uniform branch
        const float m_new = moves ? mx : m_run;
        const float m_fin = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_fin);   // 0 for a row without a reference so far, 1 if unmoved
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int c = 0; c < DB; ++c)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[c][v] *= alpha;
      }
      const float neg_m = (m_run == -INFINITY) ? 0.f : -m_run;   // (a row that has seen nothing yet: all its scores are -inf)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[nb][v] = __builtin_amdgcn_exp2f(fmaf(s[nb][v], qscale, neg_m));
    } else {
      // (mx is relative to the reference point the tile was formed with)
      const bool moves = m_run == -INFINITY ? mx > -INFINITY : mx > kLazy;
      if (__builtin_amdgcn_ballot_w64(moves) != 0) {   // wave-uniform branch
        const float m_old = (m_run == -INFINITY) ? 0.f : m_run;    // what the tile's scores are relative to
        const float m_new = moves ? m_old + mx : m_run;
        const float m_fin = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_fin);
        const float shift = m_fin - m_old;
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int c = 0; c < DB; ++c)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[c][v] *= alpha;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int v = 0; v < 16; ++v) s[nb][v] -= shift;
#pragma unroll
        for (int v = 0; v < 16; ++v) cinit[v] = -m_fin;
      }
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[nb][v] = __builtin_amdgcn_exp2f(s[nb][v]);
    }
    // lane's corner of every transposing read: key 4*hf + (lane%16)/4, dims 16*((lane/16)%2) + 4*(lane%4)
    const tr_ptr vtr = (tr_ptr)(vt + (4 * hf + ((lane & 15) >> 2)) * LDV + 16 * ((lane >> 4) & 1) + 4 * (lane & 3));
    float psum = 0.f;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        // k-slot e of this lane is key 16*t2 + 8*(e/4) + 4*hf + e%4 of block nb
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[e] = (__bf16)s[nb][8 * t2 + e];
        // row sum of the probabilities as the matrix core sees them (rounded to bf16)
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const bf16x2 pp = {pb[e], pb[e + 1]};
          psum = __builtin_amdgcn_fdot2_f32_bf16(pp, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, psum, false);
        }
#pragma unroll
        for (int c = 0; c < DB; ++c) {
          const int e0 = (nb * 32 + 16 * t2) * LDV + c * 32;   // elements past the lane's corner
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(vtr + e0 / 4);
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(vtr + (e0 + 8 * LDV) / 4);
          const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pb, o[c], 0, 0, 0);
        }
      }
    }
    l_run += psum;
  };

  // Both sets run the same program -- per tile: barrier, stage the next tile and request the one after, S = K Q^T,
  // barrier, softmax and P V -- but set 1 enters it one barrier late (and set 0 leaves it one barrier late), so the
  // k-th barrier of set 0 is the (k-1)-th of set 1 and the sets stay half a step apart: while one forms S the other
  // runs softmax and P V.  A set writes its tensor (set 0: K, set 1: V) of tile j+1 into LDS right after the first
  // barrier of its step j, at the start of the half in which it only feeds the matrix core; the half that ends in
  // softmax and P V, which sets the pace, carries no staging and no wait for global memory.
  // Visibility: K of tile j+1 is stored by set 0 after block barrier 2j and is complete before block barrier 2j+2 (the
  // fence of the storing waves' next first barrier), after which it is first read; V of tile j+1 is stored by set 1
  // after block barrier 2j+1, complete before 2j+3 and first read, by set 0, after 2j+3.
  // Reuse: the stage written in step j held tile j-1, whose last readers (both sets' S of that tile for K, both sets'
  // P V for V) finished before the barrier the write follows.
  auto stage_tile = [&](int t) __attribute__((always_inline)) {   // this set's tensor of tile t: registers -> LDS
    uint16_t* dst = reinterpret_cast<uint16_t*>(smem + (size_t)(t & 1) * Cfg::kStageBytes + stage_off_mine);
#pragma unroll
    for (int i = 0; i < NLD; ++i) *reinterpret_cast<u32x4*>(dst + (r0 + RPI * i) * ld_mine + cg * 8) = R[i];
  };
  stage_tile(0);
  if (1 < n_tiles) {
    QUOKA_ISSUE(1);
    QUOKA_RESOLVE(2);
  }
  if (set == 1) __syncthreads();   // (with the fence: V of tile 0 is complete before set 0 passes its first barrier)
  for (int j = 0; j < n_tiles; ++j) {
    __syncthreads();
    if (j + 1 < n_tiles) {
      stage_tile(j + 1);
      if (j + 2 < n_tiles) {
        QUOKA_ISSUE(j + 2);
        QUOKA_RESOLVE(j + 3);
      }
    }
    if (!computes(j)) {   // nothing visible for this wave in its share of the tile
      __builtin_amdgcn_s_barrier();
      continue;
    }
    qk(j);
    __builtin_amdgcn_s_barrier();
    softmax_pv(j);
  }
  if (set == 0) __builtin_amdgcn_s_barrier();

  // ---- merge of the two wave sets (SPLIT): set 1 hands (m, l, O) to set 0 through LDS ---------------------------
  if constexpr (SPLIT) {
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

template <int D, bool SPLIT, bool XS>
static hipError_t launch_dsx(const Dims& dm, const AttnArgs& a, hipStream_t st) {
  using Cfg = AttnCfg<D, SPLIT>;
  constexpr size_t lds = Cfg::kLdsBytes;
  static std::atomic<uint64_t> lds_done{0};
  const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&attn_bf16<D, SPLIT, XS>), lds, lds_done);
  if (e != hipSuccess) return e;
  const int nrb = dm.g * ((dm.C + 31) / 32);
  const int half = (nrb + 1) / 2;
  dim3 grid(dm.n_kv, (half + Cfg::HW - 1) / Cfg::HW, dm.b);
  AttnArgs aa = a;
  // one block is resident per compute unit: from two rounds on, neighbouring row blocks and longest ranges first
  // (measured at 512 blocks, 4096-token chunk over 131072 cached tokens: 3.5 % faster than pairing; a launch of one
  // round needs the pairing, or its last block sets the time alone)
  aa.adjacent = (long long)grid.x * grid.y * grid.z >= 2 * kComputeUnits ? 1 : 0;
  hipLaunchKernelGGL((attn_bf16<D, SPLIT, XS>), grid, dim3(2 * kSetThreads), lds, st, dm, aa);
  return hipGetLastError();
}

template <int D, bool SPLIT>
static hipError_t launch_ds(const Dims& dm, const AttnArgs& a, hipStream_t st) {
  if (dm.flags & QUOKA_ATTN_SCALE_F32) return launch_dsx<D, SPLIT, true>(dm, a, st);
  return launch_dsx<D, SPLIT, false>(dm, a, st);
}

template <int D>
static hipError_t launch_d(const Dims& dm, const AttnArgs& a, hipStream_t st) {
  const int nrb = dm.g * ((dm.C + 31) / 32);
  const long long blocks8 = (long long)dm.n_kv * (((nrb + 1) / 2 + 3) / 4) * dm.b;
  // eight row blocks per block when that still gives every compute unit a block; otherwise four, with the keys of
  // every tile split between the two wave sets
  if (blocks8 >= kComputeUnits) return launch_ds<D, false>(dm, a, st);
  return launch_ds<D, true>(dm, a, st);
}

hipError_t launch_attn_bf16(const Dims& dm, const AttnArgs& a, hipStream_t st) {
  return dm.d == 64 ? launch_d<64>(dm, a, st) : launch_d<128>(dm, a, st);
}

}  // namespace quoka
