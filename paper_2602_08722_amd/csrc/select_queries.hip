// Query sub-selection and group pre-aggregation (Alg. 1, first block and the normalise / group-mean steps;
// Sec. 3.1, 3.3).
// Memory reads are spread over the whole chip (one compute unit alone cannot pull a head's queries at more
// than a few tens of GB/s), and every kernel requests all the rows it needs before it uses the first.
//   sq_partial_sums : per (b, q-head, token tile) column sums of Q                     -> ws.part
//   sq_cosine       : per (b, q-head, token tile) mean query from the partials (fixed order, so the
//                     result is bit-reproducible), then CosSim(q_i, M_Q) for the tile   -> ws.cos
//   sq_select       : per (b, q-head) the N' lowest cosines in rank order (radix select on register-held
//                     keys + rank by counting)                                          -> q_idx
//   sq_head_select  : the three steps above in one block per (b, q-head), for batches of short chunks (the rows of
//                     a head fit the block's registers and the heads alone fill the chip)
//   sq_qbar         : per (b, KV head, r) unit-normalise the r-th retained query of each head of the
//                     group and average                                                 -> qbar
#include "common.hip.h"
#include "kernels.h"
#include "score_tile.hip.h"

namespace quoka {

constexpr int kSqTile = 64;     // tokens per tile
constexpr int kSqThreads = 256;

// ---------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kSqThreads) void sq_partial_sums(Dims dm, const T* __restrict__ q, float* __restrict__ part,
                                                             int n_tiles) {
  constexpr int CG = D / 8;              // lanes per row (8 elements each)
  constexpr int RPB = kSqThreads / CG;   // rows handled concurrently
  const int tile = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int cg = threadIdx.x % CG, rr = threadIdx.x / CG;
  const T* base = q + b * dm.qs[0] + h * dm.qs[1];
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const int t0 = tile * kSqTile;
  for (int r = rr; r < kSqTile; r += RPB) {
    const int tok = t0 + r;
    if (tok < dm.C) {
      float v[8];
      Elem<T>::load8(base + tok * dm.qs[2] + cg * 8, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += v[e];
    }
  }
  __shared__ float red[RPB][D];
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rr][cg * 8 + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0.f;
    for (int i = 0; i < RPB; ++i) s += red[i][threadIdx.x];
    part[((size_t)(b * dm.n_q + h) * n_tiles + tile) * D + threadIdx.x] = s;
  }
}

// ---------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kSqThreads) void sq_cosine(Dims dm, const T* __restrict__ q, const float* __restrict__ part,
                                                       float* __restrict__ cosv, int n_tiles) {
  constexpr int CG = D / 8;
  constexpr int RPB = kSqThreads / CG;
  const int tile = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  __shared__ float mean[D];
  __shared__ float mnorm;
  if (threadIdx.x < D) {
    const float* p = part + (size_t)(b * dm.n_q + h) * n_tiles * D + threadIdx.x;
    float s = 0.f;
    for (int i0 = 0; i0 < n_tiles; i0 += 8) {   // 8 partials requested at a time, summed in tile order
      float t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = p[(size_t)min(i0 + u, n_tiles - 1) * D];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (i0 + u < n_tiles) s += t[u];
    }
    mean[threadIdx.x] = s / (float)dm.C;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float ss = 0.f;
    for (int i = 0; i < D; ++i) ss += mean[i] * mean[i];
    mnorm = fmaxf(sqrtf(ss), kNormEps);
  }
  __syncthreads();
  const int cg = threadIdx.x % CG, rr = threadIdx.x / CG;
  float m[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) m[e] = mean[cg * 8 + e];
  const float mn = mnorm;
  const T* base = q + b * dm.qs[0] + h * dm.qs[1];
  const int t0 = tile * kSqTile;
  for (int r = rr; r < kSqTile; r += RPB) {   // uniform trip count: shuffles below stay convergent
    const int tok = t0 + r;
    const int tk = tok < dm.C ? tok : dm.C - 1;
    float v[8];
    Elem<T>::load8(base + tk * dm.qs[2] + cg * 8, v);
    float dot = 0.f, qq = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      dot += v[e] * m[e];
      qq += v[e] * v[e];
    }
    if constexpr (CG == 16) {   // a query row is exactly one 16-lane DPP row
      dot = row16_sum(dot);
      qq = row16_sum(qq);
    } else {
      dot = group_sum<CG>(dot);
      qq = group_sum<CG>(qq);
    }
    if (cg == 0 && tok < dm.C) {
      const float qn = fmaxf(sqrtf(qq), kNormEps);
      cosv[(size_t)(b * dm.n_q + h) * dm.C + tok] = dot / (qn * mn) + 0.0f;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// One block per (b, q-head): the N' lowest cosines in rank order.  Thread t keeps cosines t*IPT .. t*IPT+IPT-1
// in registers as order-preserving keys; LDS radix select (8 bits per pass, ties to the lower position) that
// starts below the leading bits all keys share (cosines to the mean sit in a narrow range), then the rank of
// every retained query among the retained ones by counting, spread over the whole block.
constexpr int kMaxKeep = 128;
constexpr int kSelThreads = 1024;

// The N' lowest keys of a block's register-held order-preserving keys, in rank order, to out[0..n_keep): radix select,
// compaction of the retained ones in position order, rank by counting.  Thread t holds positions lo .. lo+IPT-1.
template <int IPT>
__device__ __forceinline__ void select_lowest_ranked(const uint32_t (&key)[IPT], uint32_t valid, int lo, int n_keep,
                                                     RadixSelectLds& rs, uint32_t* wsum, uint32_t* sel_key,
                                                     uint32_t* sel_idx, int32_t* __restrict__ out) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  // tau: key of the n_keep-th smallest cosine; need_eq: how many elements equal to it are kept (lowest positions first)
  uint32_t tau, need_eq;
  block_radix_select<IPT, false>(key, valid, (uint32_t)n_keep, rs, &tau, &need_eq);
  // Retained queries go to LDS in position order.  One block scan carries both counts a thread needs (elements below
  // the cut in the high half, elements equal to it in the low half; both fit 16 bits since C <= 8192).
  uint32_t cnt = 0;
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    const bool in = (valid >> j) & 1u;
    cnt += (in && key[j] == tau ? 1u : 0u) + (in && key[j] < tau ? 0x10000u : 0u);
  }
  uint32_t tot;
  const uint32_t before = block_excl_scan<kSelThreads>(cnt, wsum, &tot);
  uint32_t eq_rank = before & 0xFFFFu, lt_rank = before >> 16;
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    if ((valid >> j) & 1u) {
      const uint32_t k = key[j];
      const bool lt = k < tau, eq = k == tau;
      if (lt || (eq && eq_rank < need_eq)) {   // equal cosines go to the lower positions
        const uint32_t slot = lt_rank + min(eq_rank, need_eq);
        if (slot < (uint32_t)kMaxKeep) {
          sel_key[slot] = k;
          sel_idx[slot] = (uint32_t)(lo + j);
        }
      }
      lt_rank += lt ? 1u : 0u;
      eq_rank += eq ? 1u : 0u;
    }
  }
  __syncthreads();
  // rank by counting: P consecutive lanes share one retained query and split the comparisons
  int nk2 = 1;
  while (nk2 < n_keep) nk2 <<= 1;
  const int P = kSelThreads / nk2;         // 8 .. 1024, a power of two
  const int e = tid / P, part = tid % P;
  int rank = 0;
  if (e < n_keep) {
    const uint32_t k = sel_key[e], id = sel_idx[e];
    for (int jj = part; jj < n_keep; jj += P) {
      const uint32_t kj = sel_key[jj], ij = sel_idx[jj];
      rank += (kj < k) || (kj == k && ij < id);
    }
  }
  for (int o = 1; o < P && o < 64; o <<= 1) rank += __shfl_xor(rank, o, kWave);
  if (P > 64) {   // n_keep < 16: the lanes of one query span waves; let lane 0 of each wave add through LDS
    __syncthreads();
    if (lane == 0) wsum[w] = (uint32_t)rank;
    __syncthreads();
    rank = 0;
    const int w0 = (e * P) >> 6;
    for (int i = 0; i < P / 64; ++i) rank += (int)wsum[w0 + i];
  }
  if (e < n_keep && part == 0) out[rank] = (int32_t)sel_idx[e];
}

template <int IPT>
__global__ __launch_bounds__(kSelThreads) void sq_select(Dims dm, const float* __restrict__ cosv,
                                                        int32_t* __restrict__ q_idx, int n_keep) {
  constexpr int NW = kSelThreads / 64;
  __shared__ RadixSelectLds rs;
  __shared__ uint32_t wsum[NW + 1];
  __shared__ uint32_t sel_key[kMaxKeep];
  __shared__ uint32_t sel_idx[kMaxKeep];
  const int h = blockIdx.x, b = blockIdx.y;
  const int C = dm.C;
  const float* cv = cosv + (size_t)(b * dm.n_q + h) * C;
  const int lo = threadIdx.x * IPT;
  uint32_t key[IPT];
  uint32_t valid = 0u;
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    const bool in = lo + j < C;
    key[j] = in ? okey(cv[lo + j]) : 0xFFFFFFFFu;
    valid |= (in ? 1u : 0u) << j;
  }
  select_lowest_ranked<IPT>(key, valid, lo, n_keep, rs, wsum, sel_key, sel_idx,
                            q_idx + (size_t)(b * dm.n_q + h) * n_keep);
}

// ---------------------------------------------------------------------------------------------
// Mean, cosines and selection of one (b, q-head) in one block, for chunks short enough that the block can hold the
// head's queries in registers: every row is requested at once (one memory latency; a compute unit that fetches a
// few rows per thread at a time pulls only a few tens of GB/s) and read only once.
// Column sums are formed per group of concurrently handled rows and the groups added in a fixed order, so the mean is
// bit-reproducible here too (its rounding differs from the tiled kernels' in the last bits: the two routes are
// never mixed within one call).
template <typename T>
struct Raw8;   // eight consecutive elements as loaded
template <>
struct Raw8<uint16_t> {
  u32x4 r;
  __device__ __forceinline__ void load(const uint16_t* p) { r = *reinterpret_cast<const u32x4*>(p); }
  __device__ __forceinline__ void widen(float (&v)[8]) const {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(r[i] << 16);
      v[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
    }
  }
};
template <>
struct Raw8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = *reinterpret_cast<const float4*>(p);
    b = *reinterpret_cast<const float4*>(p + 4);
  }
  __device__ __forceinline__ void widen(float (&v)[8]) const {
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};

template <typename T, int D, int NR>   // NR: rows per thread (all held in registers)
__global__ __launch_bounds__(kSelThreads) void sq_head_select(Dims dm, const T* __restrict__ q,
                                                             int32_t* __restrict__ q_idx, int n_keep) {
  constexpr int CG = D / 8;                  // lanes per row (8 elements each)
  constexpr int RPB = kSelThreads / CG;      // rows handled concurrently
  constexpr int IPT = (RPB * NR + kSelThreads - 1) / kSelThreads;   // cosines per thread in the selection
  constexpr int NW = kSelThreads / 64;
  __shared__ RadixSelectLds rs;
  __shared__ uint32_t wsum[NW + 1];
  __shared__ uint32_t sel_key[kMaxKeep];
  __shared__ uint32_t sel_idx[kMaxKeep];
  __shared__ float mean[D];
  __shared__ float mnorm;
  __shared__ float buf[RPB * D];             // column partials, then the cosines (RPB * NR <= RPB * D of them)
  const int h = blockIdx.x, b = blockIdx.y;
  const int C = dm.C;
  const int tid = threadIdx.x;
  const int cg = tid % CG, rr = tid / CG;
  const T* base = q + b * dm.qs[0] + h * dm.qs[1];
  Raw8<T> rows[NR];
#pragma unroll
  for (int u = 0; u < NR; ++u) rows[u].load(base + (size_t)min(u * RPB + rr, C - 1) * dm.qs[2] + cg * 8);
  // ---- column sums, mean, its norm ----
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int u = 0; u < NR; ++u) {
    float v[8];
    rows[u].widen(v);
    if (u * RPB + rr < C) {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += v[e];
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) buf[rr * D + cg * 8 + e] = acc[e];
  __syncthreads();
  if (tid < D) {
    float s = 0.f;
    for (int i = 0; i < RPB; ++i) s += buf[i * D + tid];
    mean[tid] = s / (float)C;
  }
  __syncthreads();
  if (tid < 64) {   // one wave: squared norm of the mean
    float ss = 0.f;
    for (int i = tid; i < D; i += 64) ss += mean[i] * mean[i];
    ss = wave64_sum(ss);
    if (tid == 0) mnorm = fmaxf(sqrtf(ss), kNormEps);
  }
  __syncthreads();   // (also: the partials in buf are dead from here on)
  float m[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) m[e] = mean[cg * 8 + e];
  const float mn = mnorm;
  // ---- cosines of the rows held in registers ----
#pragma unroll
  for (int u = 0; u < NR; ++u) {
    float v[8];
    rows[u].widen(v);
    float dot = 0.f, qq = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      dot += v[e] * m[e];
      qq += v[e] * v[e];
    }
    if constexpr (CG == 16) {
      dot = row16_sum(dot);
      qq = row16_sum(qq);
    } else {
      dot = group_sum<CG>(dot);
      qq = group_sum<CG>(qq);
    }
    const int tok = u * RPB + rr;
    if (cg == 0 && tok < C) buf[tok] = dot / (fmaxf(sqrtf(qq), kNormEps) * mn) + 0.0f;
  }
  __syncthreads();
  const int lo = tid * IPT;
  uint32_t key[IPT];
  uint32_t valid = 0u;
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    const bool in = lo + j < C;
    key[j] = in ? okey(buf[in ? lo + j : 0]) : 0xFFFFFFFFu;
    valid |= (in ? 1u : 0u) << j;
  }
  select_lowest_ranked<IPT>(key, valid, lo, n_keep, rs, wsum, sel_key, sel_idx,
                            q_idx + (size_t)(b * dm.n_q + h) * n_keep);
}

// ---------------------------------------------------------------------------------------------
// One wave per (r, kv, b): lanes own D/64 consecutive elements each.  The group's rows are all requested before
// any is used, so the kernel pays one index latency and one row latency, not g of each.
constexpr int kGroupUnroll = 8;
// RULE: where the retained positions come from.  kFromIndex: q_idx as written by the selection kernel.  The other two
// are known in closed form, so this kernel writes q_idx itself and no separate launch is needed: kIdentity keeps every
// query (C <= N_Q), kUniform takes the even stride floor(r * C / N') of the query-sampling baseline of Sec. 4.
enum { kFromIndex = 0, kIdentity = 1, kUniform = 2 };
template <typename T, int D, int RULE>
__global__ __launch_bounds__(64) void sq_qbar(Dims dm, const T* __restrict__ q, int32_t* __restrict__ q_idx,
                                             float* __restrict__ qbar, int n_keep, uint32_t* __restrict__ zero,
                                             uint32_t zero_words) {
  constexpr int EPL = D / 64;
  clear_words(zero, zero_words);   // side job of the fused call: histograms and counters of the key-selection stage
  const int r = blockIdx.x, kv = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x;
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
  for (int j0 = 0; j0 < dm.g; j0 += kGroupUnroll) {
    int tok[kGroupUnroll];
#pragma unroll
    for (int jj = 0; jj < kGroupUnroll; ++jj) {
      const int j = min(j0 + jj, dm.g - 1);
      int32_t* slot = q_idx + (size_t)(b * dm.n_q + kv * dm.g + j) * n_keep + r;
      if constexpr (RULE == kFromIndex) {
        tok[jj] = *slot;
      } else {
        tok[jj] = RULE == kIdentity ? r : (int)(((int64_t)r * dm.C) / n_keep);
        if (lane == 0) *slot = tok[jj];
      }
    }
    float v[kGroupUnroll][EPL];
#pragma unroll
    for (int jj = 0; jj < kGroupUnroll; ++jj) {
      const int j = min(j0 + jj, dm.g - 1);
      const T* row = q + b * dm.qs[0] + (size_t)(kv * dm.g + j) * dm.qs[1] + (size_t)tok[jj] * dm.qs[2];
#pragma unroll
      for (int e = 0; e < EPL; ++e) v[jj][e] = Elem<T>::load1(row + lane * EPL + e);
    }
#pragma unroll
    for (int jj = 0; jj < kGroupUnroll; ++jj) {
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) ss += v[jj][e] * v[jj][e];
      ss = wave64_sum(ss);
      const float nrm = (dm.flags & 1) ? 1.0f : fmaxf(sqrtf(ss), kNormEps);   // dot-product ablation: no normalisation
      if (j0 + jj < dm.g) {   // wave-uniform; heads are accumulated in ascending order
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += v[jj][e] / nrm;
      }
    }
  }
  float* out = qbar + ((size_t)(b * dm.n_kv + kv) * n_keep + r) * D;
#pragma unroll
  for (int e = 0; e < EPL; ++e) out[lane * EPL + e] = acc[e] / (float)dm.g;
}

// ---------------------------------------------------------------------------------------------
template <typename T, int D>
static hipError_t launch_typed(const Dims& dm, const void* q, int32_t* q_idx, float* qbar, float* ws_part,
                               float* ws_cos, hipStream_t st, uint32_t* zero, uint32_t zero_words) {
  const int n_keep = dm.n_ret < dm.C ? dm.n_ret : dm.C;
  const T* qp = static_cast<const T*>(q);
  const dim3 qgrid(n_keep, dm.n_kv, dm.b);
  if (dm.C <= dm.n_ret) {
    hipLaunchKernelGGL((sq_qbar<T, D, kIdentity>), qgrid, dim3(64), 0, st, dm, qp, q_idx, qbar, n_keep, zero, zero_words);
  } else if (dm.flags & QUOKA_SELECT_UNIFORM) {
    hipLaunchKernelGGL((sq_qbar<T, D, kUniform>), qgrid, dim3(64), 0, st, dm, qp, q_idx, qbar, n_keep, zero, zero_words);
  } else {
    const dim3 sgrid(dm.n_q, dm.b), sblock(kSelThreads);
    const int ipt = (dm.C + kSelThreads - 1) / kSelThreads;
    // One block per head for everything when the block can hold the head's queries in registers (8 rows of 8 elements
    // per thread) AND the heads alone give half the compute units a block (batches).  Measured: 256 heads of 512 tokens
    // 14.8 us against 24 us for the three launches below; with only 32 heads (1024 tokens each) one compute unit per
    // head is the slower way (20.7 against 16.5 us), so single sequences spread the two reads of Q over the whole chip.
    constexpr int kRowsPerThread = 8;
    constexpr int kRowsAtOnce = kSelThreads / (D / 8);
    if (dm.C <= kRowsAtOnce * kRowsPerThread && dm.b * dm.n_q >= 128) {
      hipLaunchKernelGGL((sq_head_select<T, D, kRowsPerThread>), sgrid, sblock, 0, st, dm, qp, q_idx, n_keep);
    } else {
      const int n_tiles = (dm.C + kSqTile - 1) / kSqTile;
      dim3 grid(n_tiles, dm.n_q, dm.b);
      hipLaunchKernelGGL((sq_partial_sums<T, D>), grid, dim3(kSqThreads), 0, st, dm, qp, ws_part, n_tiles);
      hipLaunchKernelGGL((sq_cosine<T, D>), grid, dim3(kSqThreads), 0, st, dm, qp, ws_part, ws_cos, n_tiles);
      if (ipt <= 1) {
        hipLaunchKernelGGL((sq_select<1>), sgrid, sblock, 0, st, dm, ws_cos, q_idx, n_keep);
      } else if (ipt <= 2) {
        hipLaunchKernelGGL((sq_select<2>), sgrid, sblock, 0, st, dm, ws_cos, q_idx, n_keep);
      } else if (ipt <= 4) {
        hipLaunchKernelGGL((sq_select<4>), sgrid, sblock, 0, st, dm, ws_cos, q_idx, n_keep);
      } else {
        hipLaunchKernelGGL((sq_select<8>), sgrid, sblock, 0, st, dm, ws_cos, q_idx, n_keep);
      }
    }
    hipLaunchKernelGGL((sq_qbar<T, D, kFromIndex>), qgrid, dim3(64), 0, st, dm, qp, q_idx, qbar, n_keep, zero, zero_words);
  }
  return hipGetLastError();
}

size_t select_queries_ws_floats(const Dims& dm) {
  const size_t n_tiles = (dm.C + kSqTile - 1) / kSqTile;
  return (size_t)dm.b * dm.n_q * (n_tiles * dm.d + dm.C);
}

hipError_t launch_select_queries(const Dims& dm, int dtype, const void* q, int32_t* q_idx, float* qbar, float* ws,
                                 hipStream_t st, uint32_t* zero, size_t zero_words_sz) {
  const uint32_t zero_words = (uint32_t)zero_words_sz;
  const size_t n_tiles = (dm.C + kSqTile - 1) / kSqTile;
  float* ws_part = ws;
  float* ws_cos = ws + (size_t)dm.b * dm.n_q * n_tiles * dm.d;
  if (dtype == QUOKA_F32) {
    return dm.d == 64 ? launch_typed<float, 64>(dm, q, q_idx, qbar, ws_part, ws_cos, st, zero, zero_words)
                      : launch_typed<float, 128>(dm, q, q_idx, qbar, ws_part, ws_cos, st, zero, zero_words);
  }
  return dm.d == 64 ? launch_typed<uint16_t, 64>(dm, q, q_idx, qbar, ws_part, ws_cos, st, zero, zero_words)
                    : launch_typed<uint16_t, 128>(dm, q, q_idx, qbar, ws_part, ws_cos, st, zero, zero_words);
}

}  // namespace quoka
