// Provisional key scores for long caches (Alg. 1: S = Qbar K^T with Qbar rounded to bf16, max over the query axis,
// 1/||k||), streamed at memory speed, with the histogram of the scores that the selection stage needs.
//
// Structure (one block per compute unit, a fixed grid; eight consumer waves and two producer waves):
//   * Work is the flat list of 256-key steps over (sequence, KV head, step); every block takes an equal contiguous
//     share, worked out from the device-side cache lengths, so a ragged batch leaves no compute unit idle.
//   * K travels from global memory straight into LDS (global_load_lds, 16 bytes per lane, no staging registers), one
//     step ahead of the products, through two step buffers.  The loads are issued by two producer waves that do
//     nothing else: a wave that issues more loads than the memory pipeline accepts is held at the issue until memory
//     catches up, and a wave that also had products to form would spend that time away from the matrix core
//     (measured: load issue and products then simply add up).
//   * The LDS-direct load fills 1 KiB in lane order, so rows are dense in LDS; bank conflicts are avoided by a swizzle
//     instead of padding: slot c of row r holds the row's 16-byte chunk c ^ f(r).
//   * MFMA operand plan as in the exact kernel (queries M side, keys N side), except that lane (li, hf) takes chunk
//     ks + KS*hf of its key in k-step ks (the contraction index may be permuted freely as long as the query operand
//     uses the same permutation); with the swizzle above this keeps every ds_read_b128 conflict-free.
//   * A wave owns one query block and QB of the step's eight 32-key blocks; the operand reads of the next key block
//     are issued before the products of the current one, and every key block runs as two MFMA chains.
//   * A step's scores are finished one step later, under the next step's barrier; each finished score is counted in a
//     per-block LDS histogram (4096 equal bins of [-1, 1], two 16-bit counters per word) that is flushed with integer
//     atomics when the block leaves a head.
#include "common.hip.h"
#include "kernels.h"
#include "score_tile.hip.h"
#include "select_ws.hip.h"

namespace quoka {

constexpr int kStWaves = 8;           // consumer waves: products, maxima, norms, scores
constexpr int kStProducers = 2;       // producer waves: loads only
constexpr int kStThreads = 64 * (kStWaves + kStProducers);
constexpr int kStConsumerThreads = 64 * kStWaves;
constexpr int kStKeys = 256;          // keys per step
constexpr int kStRing = 2;            // step buffers
constexpr int kStGrid = 256;          // one block per compute unit of an MI355X
constexpr int kStFlushSteps = 255;    // 255 * 256 keys < 2^16: a 16-bit bin counter cannot overflow between flushes

template <int D, int QB>
struct StreamCfg {
  static constexpr int KS = D / 16;                    // MFMA k-steps
  static constexpr int CPR = D / 8;                    // 16-byte chunks per key row
  static constexpr int ROW_B = D * 2;                  // bytes per key row (dense in LDS)
  static constexpr int STEP_B = kStKeys * ROW_B;       // bytes per step
  static constexpr int RPI = 1024 / ROW_B;             // rows one wave-wide load covers
  static constexpr int IPP = STEP_B / 1024 / kStProducers;   // wave-wide loads per producer wave and step
  static constexpr int NP = 16 / RPI;                  // distinct swizzle patterns of a wave-wide load (by load % NP)
  static constexpr int FSH = CPR == 16 ? 0 : 1;        // swizzle f(r) = (r >> FSH) % CPR: 16 consecutive rows hit
                                                       // 16 different 16-byte columns of the 256-byte bank line
  static constexpr int UPW = QB;                       // 32-key blocks per wave and step (QB * 8 units on 8 waves)
  static constexpr int KB_STEP = kStWaves / QB;        // this wave's key blocks: w / QB + i * KB_STEP
  static constexpr int NKS = KS / QB;                  // k-steps whose squares this wave adds up for the norms
  static constexpr size_t kLdsBytes =
      (size_t)kStRing * STEP_B + (kSelBins / 2) * 4 + 2 * QB * kStKeys * 4 /*maxima*/ + 2 * QB * kStKeys * 4 /*norms*/;
};

// LDS[m0 + lane * 16 .. + 16] <- 16 bytes at base + voff (per lane); completion is counted by vmcnt
__device__ __forceinline__ void dma16(const char* base, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(base)
               : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int D, int QB>
__global__ __launch_bounds__(kStThreads, 1) void score_stream(Dims dm, const float* __restrict__ qbar,
                                                             const uint16_t* __restrict__ kc,
                                                             const int32_t* __restrict__ kv_lens,
                                                             float* __restrict__ scores, uint32_t* __restrict__ hist_ws,
                                                             int n_keep) {
  using Cfg = StreamCfg<D, QB>;
  constexpr int KS = Cfg::KS, CPR = Cfg::CPR, ROW_B = Cfg::ROW_B, STEP_B = Cfg::STEP_B, RPI = Cfg::RPI, IPP = Cfg::IPP,
                NP = Cfg::NP, FSH = Cfg::FSH, UPW = Cfg::UPW, KB_STEP = Cfg::KB_STEP, NKS = Cfg::NKS;
  extern __shared__ __align__(1024) unsigned char smem[];
  unsigned char* ring = smem;
  uint32_t* lh = reinterpret_cast<uint32_t*>(smem + (size_t)kStRing * STEP_B);   // [kSelBins / 2], two counters a word
  float* smax = reinterpret_cast<float*>(lh + kSelBins / 2);                      // [2][QB][kStKeys]
  float* ssq = smax + 2 * QB * kStKeys;                                           // [2][QB][kStKeys] partial sums
  const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)ring;

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, hf = lane >> 5;
  const bool producer = w >= kStWaves;
  const int qb = w % QB;        // a consumer wave's query block
  const int kb0 = (w % kStWaves) / QB;   // and its first key block

  for (int i = tid; i < kSelBins / 2; i += kStThreads) lh[i] = 0u;

  // ---- this block's share of the flat step list ----
  long long total = 0;
  for (int b = 0; b < dm.b; ++b) {
    const int T = max(0, min(kv_lens[b], dm.T_max));
    total += (long long)dm.n_kv * ((T + kStKeys - 1) / kStKeys);
  }
  long long cur = total * blockIdx.x / gridDim.x;
  const long long end = total * (blockIdx.x + 1) / gridDim.x;
  int sb = 0;              // sequence that holds `cur`
  long long acc_steps = 0; // steps of the sequences before sb

  // Producer lanes: wave-wide load q of a step covers rows q*RPI .. +RPI; this lane's row inside it and its swizzled
  // chunk, which depends on q only through q % NP.
  const int ld_row = lane / CPR;
  uint32_t ld_chunk[NP];
#pragma unroll
  for (int pch = 0; pch < NP; ++pch) ld_chunk[pch] = (uint32_t)(((lane % CPR) ^ (((pch * RPI + ld_row) >> FSH) % CPR)) * 16);
  // operand reads: byte offset of this lane's chunk of key row li of a 32-key block, per k-step
  uint32_t rd_off[KS];
  {
    const int y = (KS * hf) ^ ((li >> FSH) % CPR);   // rows of later 32-key blocks have the same f (32 % 16 == 0)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) rd_off[ks] = (uint32_t)(li * ROW_B + ((ks ^ y) * 16));
  }

  while (cur < end) {
    // ---- locate (sequence, head, first step) of the segment and its length ----
    int T, nb;
    for (;;) {
      T = max(0, min(kv_lens[sb], dm.T_max));
      nb = (T + kStKeys - 1) / kStKeys;
      if (cur < acc_steps + (long long)dm.n_kv * nb) break;
      acc_steps += (long long)dm.n_kv * nb;
      ++sb;
    }
    const int rem = (int)(cur - acc_steps);
    const int kv = rem / nb, step0 = rem % nb;
    const int n = (int)min((long long)(nb - step0), end - cur);
    cur += n;
    const int head = sb * dm.n_kv + kv;
    const char* kbase = reinterpret_cast<const char*>(kc + sb * dm.kvs[0] + kv * dm.kvs[1]);
    const uint32_t row_bytes = (uint32_t)dm.kvs[2] * 2u;
    float* sc = scores + (size_t)head * dm.T_max;
    const int key0 = step0 * kStKeys;

    // per-lane byte offsets inside a wave-wide load (the same for every load that lies inside the cache extent)
    uint32_t ld_off[NP];
#pragma unroll
    for (int pch = 0; pch < NP; ++pch) ld_off[pch] = (uint32_t)ld_row * row_bytes + ld_chunk[pch];

    auto issue_step = [&](int j) __attribute__((always_inline)) {   // producer waves only
      const int pw = w - kStWaves;
      const int row0 = key0 + j * kStKeys;
      const bool inside = row0 + kStKeys <= dm.T_max;
#pragma unroll 4
      for (int i = 0; i < IPP; ++i) {
        const int q = pw * IPP + i;
        const uint32_t dst = ring_lds + (uint32_t)((j % kStRing) * STEP_B + q * 1024);
        // (a head's rows span less than 4 GiB: checked on the host)
        const char* qbase = kbase + (size_t)(row0 + q * RPI) * row_bytes;
        if (inside) {
          dma16(qbase, ld_off[i % NP], dst);   // (pw * IPP is a multiple of NP)
        } else {
          // the step reaches past the cache extent: rows are clamped to allocated memory (their scores are not used)
          const uint32_t r = (uint32_t)min(q * RPI + ld_row, dm.T_max - 1 - row0);   // relative to the step's first row
          dma16(kbase + (size_t)row0 * row_bytes, r * row_bytes + ld_chunk[i % NP], dst);
        }
      }
    };
    if (producer) {
      issue_step(0);
      wait_vmcnt<0>();
    }

    // query operand of this wave: rows qb*32 .. +32 of the head's Qbar, rounded to bf16, chunk ks + KS*hf per k-step
    bf16x8 qa[KS];
    if (!producer) {
      float d2 = 0.f;
      const int r = min(qb * 32 + li, n_keep - 1);   // padding rows repeat a real query: the max is unchanged
      const float* qrow = qbar + ((size_t)head * n_keep + r) * D;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const float4 x0 = *reinterpret_cast<const float4*>(qrow + (ks + KS * hf) * 8);
        const float4 x1 = *reinterpret_cast<const float4*>(qrow + (ks + KS * hf) * 8 + 4);
        const float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          qa[ks][e] = (__bf16)x[e];
          const float dlt = x[e] - (float)qa[ks][e];
          d2 += dlt * dlt;
        }
      }
      // the error bound of these provisional scores: the largest distance between a row of Qbar and its bf16 rounding
      // (squared; non-negative floats order like their bit patterns, so an integer max collects it per head)
      d2 += other_half(d2);
      d2 = wave64_max(d2);
      if (hist_ws != nullptr && lane == 0)
        atomicMax(hist_ws + (size_t)head * (kSelBins + kSelMeta) + kSelBins + kMetaEps2, __float_as_uint(d2));
    }

    auto finish = [&](int j) __attribute__((always_inline)) {
      if (tid < kStKeys) {
        const int key = key0 + j * kStKeys + tid;
        if (key < T) {
          const float* sm = smax + (j & 1) * QB * kStKeys;
          const float* sq = ssq + (j & 1) * QB * kStKeys;
          float m = sm[tid], s2 = sq[tid];
#pragma unroll
          for (int q = 1; q < QB; ++q) {
            m = fmaxf(m, sm[q * kStKeys + tid]);
            s2 += sq[q * kStKeys + tid];
          }
          const float v = m / fmaxf(sqrtf(s2), kNormEps) + 0.0f;
          sc[key] = v;
          if (hist_ws != nullptr) {
            const int bin = score_bin(v);
            atomicAdd(&lh[bin >> 1], 1u << ((bin & 1) * 16));
          }
        }
      }
    };

    auto flush_hist = [&]() __attribute__((always_inline)) {
      uint32_t* gh = hist_ws + (size_t)head * (kSelBins + kSelMeta);
      for (int i = tid; i < kSelBins / 2; i += kStThreads) {
        const uint32_t v = lh[i];
        if (v) {
          if (v & 0xFFFFu) atomicAdd(&gh[2 * i], v & 0xFFFFu);
          if (v >> 16) atomicAdd(&gh[2 * i + 1], v >> 16);
          lh[i] = 0u;
        }
      }
    };

    auto compute = [&](int j) __attribute__((always_inline)) {
      const unsigned char* tl = ring + (size_t)(j % kStRing) * STEP_B;
      float* smax_g = smax + (j & 1) * QB * kStKeys + qb * kStKeys;
      float* ssq_g = ssq + (j & 1) * QB * kStKeys + qb * kStKeys;
      bf16x8 kop[2][KS];
      auto read_ops = [&](int u, bf16x8 (&dst)[KS]) __attribute__((always_inline)) {
        const unsigned char* kp = tl + (kb0 + u * KB_STEP) * 32 * ROW_B;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) dst[ks] = *reinterpret_cast<const bf16x8*>(kp + rd_off[ks]);
      };
      read_ops(0, kop[0]);
#pragma unroll
      for (int u = 0; u < UPW; ++u) {
        // the next key block's operands are requested before this one's products are issued
        if (u + 1 < UPW) read_ops(u + 1, kop[(u + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
        f32x16 c0 = {0}, c1 = {0};   // two chains (even / odd k-steps): a single dependent chain idles the matrix core
#pragma unroll
        for (int ks = 0; ks < KS; ks += 2) {
          c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[ks], kop[u & 1][ks], c0, 0, 0, 0);
          c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[ks + 1], kop[u & 1][ks + 1], c1, 0, 0, 0);
        }
        // this wave's share of the squared norms: the k-steps qb*NKS .. +NKS of both half waves (the waves that hold
        // the other query blocks of the same keys add the rest)
        float ss = 0.f;
#pragma unroll
        for (int k2 = 0; k2 < NKS; ++k2) {
          bf16x8 kv8 = kop[u & 1][k2];
#pragma unroll
          for (int q = 1; q < QB; ++q)
            if (q == qb) kv8 = kop[u & 1][q * NKS + k2];   // (wave-uniform selection among QB <= 4 candidates)
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            const bf16x2_t pr = {kv8[e], kv8[e + 1]};
            ss = __builtin_amdgcn_fdot2_f32_bf16(pr, pr, ss, false);
          }
        }
        ss += other_half(ss);
        float m = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) m = fmaxf(m, c0[v] + c1[v]);
        m = fmaxf(m, other_half(m));
        if (hf == 0) {
          const int k = (kb0 + u * KB_STEP) * 32 + li;
          smax_g[k] = m;
          ssq_g[k] = ss;
        }
      }
    };

    int since_flush = 0;
    for (int j = 0; j < n; ++j) {
      // One barrier per step: step j has landed (its producers waited for their loads before arriving), the maxima
      // and norms of step j-1 are published, and everybody has finished reading the buffer of step j-1, which the
      // next load overwrites.
      __syncthreads();
      if (producer) {
        if (j + 1 < n) issue_step(j + 1);
        wait_vmcnt<0>();
      } else {
        compute(j);
        if (j > 0) finish(j - 1);
      }
      if (hist_ws != nullptr && ++since_flush >= kStFlushSteps) {   // block-uniform
        __syncthreads();
        flush_hist();
        since_flush = 0;
      }
    }
    __syncthreads();
    finish(n - 1);
    __syncthreads();
    if (hist_ws != nullptr) flush_hist();   // leave the head: flush the occupied bins
    __syncthreads();                        // buffers, maxima and the histogram are free for the next segment
  }
}

template <int D, int QB>
static hipError_t launch_stream_q(const Dims& dm, const float* qbar, const void* kc, const int32_t* kv_lens,
                                  float* scores, uint32_t* hist_ws, int n_keep, hipStream_t st) {
  using Cfg = StreamCfg<D, QB>;
  static std::atomic<uint64_t> lds_done{0};
  const hipError_t e =
      ensure_dynamic_lds(reinterpret_cast<const void*>(&score_stream<D, QB>), Cfg::kLdsBytes, lds_done);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((score_stream<D, QB>), dim3(kStGrid), dim3(kStThreads), Cfg::kLdsBytes, st, dm, qbar,
                     static_cast<const uint16_t*>(kc), kv_lens, scores, hist_ws, n_keep);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_stream_d(const Dims& dm, const float* qbar, const void* kc, const int32_t* kv_lens,
                                  float* scores, uint32_t* hist_ws, int n_keep, hipStream_t st) {
  const int qblocks = (n_keep + 31) / 32;
  if (qblocks <= 1) return launch_stream_q<D, 1>(dm, qbar, kc, kv_lens, scores, hist_ws, n_keep, st);
  if (qblocks == 2) return launch_stream_q<D, 2>(dm, qbar, kc, kv_lens, scores, hist_ws, n_keep, st);
  return launch_stream_q<D, 4>(dm, qbar, kc, kv_lens, scores, hist_ws, n_keep, st);
}

// Provisional (one bf16 term) cosine / max scores of every cached key; with `hist_ws` (the zeroed head of the
// selection workspace) also their per-head histogram.
hipError_t launch_score_stream(const Dims& dm, const float* qbar, const void* k_cache, const int32_t* kv_lens,
                               float* scores, uint32_t* hist_ws, hipStream_t st) {
  if (dm.T_max <= 0) return hipSuccess;
  const int n_keep = dm.n_ret < dm.C ? dm.n_ret : dm.C;
  return dm.d == 64 ? launch_stream_d<64>(dm, qbar, k_cache, kv_lens, scores, hist_ws, n_keep, st)
                    : launch_stream_d<128>(dm, qbar, k_cache, kv_lens, scores, hist_ws, n_keep, st);
}

}  // namespace quoka
