// Attention for decode-sized chunks (Sec. 4.4: generation uses the same selection with B_CP = 1; Alg. 1 keeps every
// query when B_CP <= N_Q): the g * C query rows of one KV head fit one 32-row MFMA block, so the work is split over
// the KEY axis instead (split-KV): block (split, kv, b) attends its rows over one contiguous range of the key list
// [gathered cache rows | chunk rows] and writes an un-normalised partial (m, l, O); a second kernel merges the
// partials with the usual log-sum-exp rescale (Eq. 2-3 are unchanged, only the summation is regrouped).
//
// Rows: row r = c * g + j is chunk token c of q-head kv * g + j.  Keys: list slot n < n_cache is a cache row
// (k_idx[n] on the sparse path, n itself on the dense path), slot n_cache + p is chunk row p, visible to token c
// iff p <= c.  A tile is 128 list slots; wave w of the block takes slots 32 w .. 32 w + 31 of every tile of the
// block's range and keeps its own running (m, l, O), merged through LDS at the end of the block.
// MFMA operand plan as in the prefill kernel: S^T = K Q^T (query rows on lanes), O^T += V^T P^T with V^T fetched
// by the transposing LDS read.
#include "common.hip.h"
#include "kernels.h"

namespace quoka {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef s16x4 __attribute__((address_space(3))) * tr_ptr;

constexpr int kDcThreads = 256;
constexpr int kDcTile = 128;   // list slots per staged tile (32 per wave)

template <int D>
struct DecodeCfg {
  static constexpr int KS = D / 16;
  static constexpr int LD = D + 8;        // K rows: 16 bytes of padding (conflict-free b128 reads)
  static constexpr int LDV = D + 32;      // V rows: 64 bytes apart modulo 256 (transposing reads)
  static constexpr int CG = D / 8;
  static constexpr int RPI = kDcThreads / CG;
  static constexpr int NLD = kDcTile / RPI;
  static constexpr int DB = D / 32;
  static constexpr size_t kKBytes = (size_t)kDcTile * LD * 2;
  static constexpr size_t kStageBytes = kKBytes + (size_t)kDcTile * LDV * 2;
  static constexpr size_t kLdsBytes = 2 * kStageBytes;
  static constexpr int REC = 2 + D;       // floats per row of a partial: m, l, O[D]
};

// part: [b, n_kv, n_splits, 32 rows, REC] float32
template <int D>
__global__ __launch_bounds__(kDcThreads, 2) void attn_decode_bf16(Dims dm, AttnArgs a, float* __restrict__ part,
                                                                  int n_splits, int slots_per_split) {
  using Cfg = DecodeCfg<D>;
  constexpr int KS = Cfg::KS, LD = Cfg::LD, LDV = Cfg::LDV, CG = Cfg::CG, RPI = Cfg::RPI, NLD = Cfg::NLD, DB = Cfg::DB,
                REC = Cfg::REC;
  extern __shared__ __align__(16) unsigned char smem[];
  const int split = blockIdx.x, kv = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, hf = lane >> 5;
  const int C = dm.C, g = dm.g;
  const int n_rows = C * g;   // <= 32, checked by the launcher

  const bool sparse = a.k_idx != nullptr;
  int n_cache = sparse ? min(a.n_cache[b * dm.n_kv + kv], dm.B_max) : min(a.n_cache[b], dm.T_max);
  n_cache = max(n_cache, 0);
  const int n_keys = n_cache + C;
  const int s_begin = split * slots_per_split;
  const int s_end = min(s_begin + slots_per_split, n_keys);
  float* my_part = part + ((size_t)(b * dm.n_kv + kv) * n_splits + split) * 32 * REC;
  if (s_begin >= s_end) {   // block-uniform: an empty range contributes the neutral partial
    for (int i = tid; i < 32 * REC; i += kDcThreads) my_part[i] = (i % REC == 0) ? -INFINITY : 0.f;
    return;
  }
  const int n_tiles = (s_end - s_begin + kDcTile - 1) / kDcTile;

  const char* kcache = reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.k_cache) + b * dm.kvs[0] + kv * dm.kvs[1]);
  const char* vcache = reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.v_cache) + b * dm.kvs[0] + kv * dm.kvs[1]);
  const char* kchunk = reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.k_chunk) + b * dm.cks[0] + kv * dm.cks[1]);
  const char* vchunk = reinterpret_cast<const char*>(static_cast<const uint16_t*>(a.v_chunk) + b * dm.cks[0] + kv * dm.cks[1]);
  const int32_t* kidx = sparse ? a.k_idx + (size_t)(b * dm.n_kv + kv) * dm.B_max : nullptr;
  const uint32_t cache_row_bytes = (uint32_t)dm.kvs[2] * 2u, chunk_row_bytes = (uint32_t)dm.cks[2] * 2u;
  const uint64_t k_cache_u = reinterpret_cast<uint64_t>(kcache), v_cache_u = reinterpret_cast<uint64_t>(vcache);
  const uint64_t k_chunk_delta = reinterpret_cast<uint64_t>(kchunk) - k_cache_u;   // modulo 2^64
  const uint64_t v_chunk_delta = reinterpret_cast<uint64_t>(vchunk) - v_cache_u;

  // Q operand: row li -> (token li / g, head li % g); padding rows repeat row 0 and are never stored
  const int row = li < n_rows ? li : 0;
  const int tok = row / g, hj = row % g;
  bf16x8 qreg[KS];
  {
    const uint16_t* qrow = static_cast<const uint16_t*>(a.q) + b * dm.qs[0] + (size_t)(kv * g + hj) * dm.qs[1] +
                           (size_t)tok * dm.qs[2] + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
  }

  const int cg = tid % CG, r0 = tid / CG;
  u32x4 RK[NLD], RV[NLD];
  // all rows of a tile are requested together: indices first (one latency), then the rows (one latency)
  auto issue = [&](int t) __attribute__((always_inline)) {
    const int base = s_begin + t * kDcTile;
    // addresses as integers (cache base, plus the distance to the chunk tensor for chunk rows): a per-lane choice
    // between two pointers would be kept as a table in scratch memory
    uint64_t ka[NLD], va[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int n = min(base + r0 + RPI * i, s_end - 1);   // tail slots repeat a real row; they are masked below
      const bool from_cache = n < n_cache;
      int src = from_cache ? n : n - n_cache;
      if (from_cache && sparse) src = (int)min((uint32_t)kidx[n], (uint32_t)(dm.T_max - 1));   // a malformed list cannot leave the cache
      const uint64_t off = (uint64_t)((uint32_t)src * (from_cache ? cache_row_bytes : chunk_row_bytes) + (uint32_t)cg * 16u);
      ka[i] = k_cache_u + (from_cache ? 0ull : k_chunk_delta) + off;
      va[i] = v_cache_u + (from_cache ? 0ull : v_chunk_delta) + off;
    }
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      RK[i] = *reinterpret_cast<const u32x4*>(ka[i]);
      RV[i] = *reinterpret_cast<const u32x4*>(va[i]);
    }
  };
  issue(0);

  f32x16 o[DB];
#pragma unroll
  for (int c = 0; c < DB; ++c)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[c][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sl2 = 1.4426950408889634f / sqrtf((float)D);

  for (int t = 0; t < n_tiles; ++t) {
    uint16_t* kt = reinterpret_cast<uint16_t*>(smem + (size_t)(t & 1) * Cfg::kStageBytes);
    uint16_t* vt = reinterpret_cast<uint16_t*>(smem + (size_t)(t & 1) * Cfg::kStageBytes + Cfg::kKBytes);
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int rl = r0 + RPI * i;
      *reinterpret_cast<u32x4*>(kt + rl * LD + cg * 8) = RK[i];
      *reinterpret_cast<u32x4*>(vt + rl * LDV + cg * 8) = RV[i];
    }
    __syncthreads();   // tile t visible; the other stage was last read before the previous barrier
    if (t + 1 < n_tiles) issue(t + 1);

    const int slot0 = s_begin + t * kDcTile + w * 32;   // this wave's 32 slots
    if (slot0 >= s_end) continue;                       // wave-uniform
    // ---- S^T = K Q^T ----
    f32x16 s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
    const uint16_t* kp = kt + (w * 32 + li) * LD + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 kop = *reinterpret_cast<const bf16x8*>(kp + ks * 16);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop, qreg[ks], s, 0, 0, 0);
    }
    // ---- mask: slots past the range; chunk rows in the token's future ----
    // slot n is visible iff n < s_end and (it is a cache slot or its chunk position n - n_cache is <= tok),
    // i.e. iff n < min(s_end, n_cache + tok + 1): one lane-private limit, as in the prefill kernel
    const int limit = min(s_end, n_cache + tok + 1) - slot0;   // keys kk < limit of this wave's 32 are visible
    if (slot0 + 32 > min(s_end, n_cache)) {   // wave-uniform: the block of 32 touches the tail or the chunk rows
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int kk = 8 * (v / 4) + 4 * hf + (v % 4);
        if (kk >= limit) s[v] = -INFINITY;
      }
    }
    // ---- online softmax ----
    float mx = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[v]);
    mx = fmaxf(mx, other_half(mx)) * sl2;
    // the reference point only moves when the tile maximum exceeds it by more than 2^8 (as in the prefill kernel)
    constexpr float kLazy = 8.0f;
    if (__builtin_amdgcn_ballot_w64(mx > m_run + kLazy) != 0) {   // wave-uniform branch
      const float m_new = (mx > m_run + kLazy) ? mx : m_run;
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
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = __builtin_amdgcn_exp2f(fmaf(s[v], sl2, -m_use));
    // ---- O^T += V^T P^T ----
    const tr_ptr vtr = (tr_ptr)(vt + (w * 32 + 4 * hf + ((lane & 15) >> 2)) * LDV + 16 * ((lane >> 4) & 1) + 4 * (lane & 3));
    float psum = 0.f;
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      bf16x8 pb;
#pragma unroll
      for (int e = 0; e < 8; ++e) pb[e] = (__bf16)s[8 * t2 + e];
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        const bf16x2 pp = {pb[e], pb[e + 1]};
        psum = __builtin_amdgcn_fdot2_f32_bf16(pp, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, psum, false);
      }
#pragma unroll
      for (int c = 0; c < DB; ++c) {
        const int e0 = (16 * t2) * LDV + c * 32;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(vtr + e0 / 4);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(vtr + (e0 + 8 * LDV) / 4);
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pb, o[c], 0, 0, 0);
      }
    }
    l_run += psum;
  }

  // ---- merge the four waves' partials through LDS, then write the block's partial ----------------------------
  const float l_wave = l_run + other_half(l_run);
  __syncthreads();   // the tile buffers may be reused
  float* mg = reinterpret_cast<float*>(smem);   // [4 waves][32 rows][REC]
  {
    float* rec = mg + ((size_t)w * 32 + li) * REC;
    if (hf == 0) {
      rec[0] = m_run;
      rec[1] = l_wave;
    }
#pragma unroll
    for (int c = 0; c < DB; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) rec[2 + 32 * c + 8 * (v / 4) + 4 * hf + (v % 4)] = o[c][v];
  }
  __syncthreads();
  for (int i = tid; i < 32 * REC; i += kDcThreads) {
    const int r = i / REC, e = i % REC;
    float m = -INFINITY;
#pragma unroll
    for (int u = 0; u < 4; ++u) m = fmaxf(m, mg[((size_t)u * 32 + r) * REC]);
    float acc = 0.f;
    if (e == 0) {
      acc = m;
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float mu = mg[((size_t)u * 32 + r) * REC];
        const float wgt = (mu == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mu - m);
        acc += wgt * mg[((size_t)u * 32 + r) * REC + e];
      }
    }
    my_part[i] = acc;
  }
}

// One block per (row, kv, b).  The splits' (m, l) go through LDS once; then thread (dim e, split group sg) adds up the
// O partials of its splits (independent, coalesced loads, unrolled), and the groups are combined through LDS.
// The summation order is fixed by the indices alone, so the result does not depend on scheduling.
constexpr int kMaxSplits = 64;
template <int D>
__global__ __launch_bounds__(kDcThreads) void attn_decode_merge(Dims dm, AttnArgs a, const float* __restrict__ part,
                                                                int n_splits) {
  constexpr int REC = DecodeCfg<D>::REC;
  constexpr int NG = kDcThreads / D;   // split groups
  __shared__ float wgt[kMaxSplits];
  __shared__ float red[NG][D];
  __shared__ float s_m, s_l;
  const int r = blockIdx.x, kv = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const float* base = part + ((size_t)(b * dm.n_kv + kv) * n_splits * 32 + r) * REC;   // split s is s * 32 * REC further
  const size_t sstride = (size_t)32 * REC;
  float m_s = -INFINITY, l_s = 0.f;
  if (tid < n_splits) {
    m_s = base[tid * sstride];
    l_s = base[tid * sstride + 1];
  }
  if (tid < 64) {   // n_splits <= 64: one wave holds all of them
    const float m = wave64_max(m_s);
    const float w = (m_s == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_s - m);
    const float l = wave64_sum(w * l_s);
    if (tid < n_splits) wgt[tid] = w;
    if (tid == 0) {
      s_m = m;
      s_l = l;
    }
  }
  __syncthreads();
  const int e = tid % D, sg = tid / D;
  float acc = 0.f;
  for (int s0 = sg; s0 < n_splits; s0 += 8 * NG) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int sp = min(s0 + u * NG, n_splits - 1);
      v[u] = base[sp * sstride + 2 + e];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (s0 + u * NG < n_splits) acc += wgt[s0 + u * NG] * v[u];
  }
  red[sg][e] = acc;
  __syncthreads();
  if (tid < D) {
    float o = red[0][tid];
#pragma unroll
    for (int g2 = 1; g2 < NG; ++g2) o += red[g2][tid];
    const int tok = r / dm.g, h = kv * dm.g + r % dm.g;
    uint16_t* orow = static_cast<uint16_t*>(a.out) + b * dm.os[0] + h * dm.os[1] + (size_t)tok * dm.os[2];
    orow[tid] = (uint16_t)f32_to_bf16_bits(o / s_l);
    if (tid == 0 && a.lse != nullptr) a.lse[(size_t)(b * dm.n_q + h) * dm.C + tok] = (s_m + log2f(s_l)) * 0.6931471805599453f;
  }
}

// ---------------------------------------------------------------------------------------------
bool attn_decode_applies(const Dims& dm) { return dm.C * dm.g <= 32; }

static int decode_splits(const Dims& dm, bool sparse) {
  const long long max_keys = (long long)(sparse ? dm.B_max : dm.T_max) + dm.C;
  const long long tiles = (max_keys + kDcTile - 1) / kDcTile;
  long long n = (tiles + 7) / 8;                                   // about eight tiles per split ...
  const long long fill = (256 + (long long)dm.b * dm.n_kv - 1) / ((long long)dm.b * dm.n_kv);
  if (n < fill) n = fill < tiles ? fill : tiles;                   // ... but enough splits to give every CU a block
  n = n < 1 ? 1 : (n > kMaxSplits ? kMaxSplits : n);
  return (int)n;
}

size_t attn_decode_ws_floats(const Dims& dm) {
  if (dm.g > 32) return 0;
  // Independent of the chunk length (a prompt's last chunk may be decode-sized when the others are not), and sized
  // for the dense path (the larger key list), so one workspace serves every call made with this shape.
  return (size_t)dm.b * dm.n_kv * decode_splits(dm, false) * 32 * (2 + dm.d);
}

template <int D>
static hipError_t launch_decode_d(const Dims& dm, const AttnArgs& a, float* part, hipStream_t st) {
  using Cfg = DecodeCfg<D>;
  static std::atomic<uint64_t> lds_done{0};
  const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(&attn_decode_bf16<D>), Cfg::kLdsBytes, lds_done);
  if (e != hipSuccess) return e;
  const bool sparse = a.k_idx != nullptr;
  const int n_splits = decode_splits(dm, sparse);
  const long long max_keys = (long long)(sparse ? dm.B_max : dm.T_max) + dm.C;
  int sps = (int)((max_keys + n_splits - 1) / n_splits);
  sps = (sps + kDcTile - 1) / kDcTile * kDcTile;
  hipLaunchKernelGGL((attn_decode_bf16<D>), dim3(n_splits, dm.n_kv, dm.b), dim3(kDcThreads), Cfg::kLdsBytes, st, dm, a,
                     part, n_splits, sps);
  hipLaunchKernelGGL((attn_decode_merge<D>), dim3(dm.C * dm.g, dm.n_kv, dm.b), dim3(kDcThreads), 0, st, dm, a, part,
                     n_splits);
  return hipGetLastError();
}

hipError_t launch_attn_decode_bf16(const Dims& dm, const AttnArgs& a, float* part, hipStream_t st) {
  return dm.d == 64 ? launch_decode_d<64>(dm, a, part, st) : launch_decode_d<128>(dm, a, part, st);
}

}  // namespace quoka
