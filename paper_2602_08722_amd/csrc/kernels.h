// Internal launcher interface between the C-ABI layer (api.hip) and the kernel translation units.
#pragma once
#include <atomic>
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "common.hip.h"

namespace quoka {

// Kernels that use more than 64 KiB of dynamic LDS need the limit raised once per function and device.  `done` is a
// per-function bit mask over device ordinals (a function-local static of the caller); the attribute call is
// idempotent, so two threads racing through it are harmless, and the mask itself is atomic.
inline hipError_t ensure_dynamic_lds(const void* func, size_t bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t{1} << dev) : 0;   // ordinals beyond 63: set it every time
  if (bit != 0 && (done.load(std::memory_order_acquire) & bit) != 0) return hipSuccess;
  e = hipFuncSetAttribute(func, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return e;
  done.fetch_or(bit, std::memory_order_release);
  return hipSuccess;
}

// --- query sub-selection (select_queries.hip) -------------------------------------------------
size_t select_queries_ws_floats(const Dims& dm);
// `zero` / `zero_words`: optional side job for the fused call -- the last launch clears that many 32-bit words (what
// the key-selection stage that follows needs cleared).
hipError_t launch_select_queries(const Dims& dm, int dtype, const void* q, int32_t* q_idx, float* qbar, float* ws,
                                 hipStream_t st, uint32_t* zero = nullptr, size_t zero_words = 0);

// --- key scoring (score_keys.hip) ---------------------------------------------------------------
// `zero` / `zero_words`: optional side job for the fused call -- the scoring blocks clear that many 32-bit words (the
// histograms the multi-block top-k that follows would otherwise clear with a launch of its own).
hipError_t launch_score_keys(const Dims& dm, int dtype, const float* qbar, const void* k_cache, const int32_t* kv_lens,
                             float* scores, hipStream_t st, uint32_t* zero = nullptr, size_t zero_words = 0);

// --- top-B key selection (topk_keys.hip) ----------------------------------------------------------
size_t topk_ws_words(const Dims& dm);
// `ws_is_zero`: the workspace words (topk_ws_words) have already been cleared on this stream.
hipError_t launch_topk_keys(const Dims& dm, const float* scores, const int32_t* kv_lens, const int32_t* budgets,
                            int32_t* k_idx, int32_t* k_cnt, uint32_t* ws, hipStream_t st, bool ws_is_zero = false);

// --- scoring + top-B as one stage for long caches (select_keys.hip) --------------------------------
// Provisional one-term scores, exact re-scoring of the keys near the cut, ordered emission: the same index lists as
// launch_score_keys followed by launch_topk_keys.  `ws_is_zero`: the first select_keys_zero_words words of the
// workspace have already been cleared on this stream.
hipError_t launch_score_stream(const Dims& dm, const float* qbar, const void* k_cache, const int32_t* kv_lens,
                               float* scores, uint32_t* hist_ws, hipStream_t st);
bool select_keys_two_pass_applies(const Dims& dm, int dtype);
size_t select_keys_ws_words(const Dims& dm);
size_t select_keys_zero_words(const Dims& dm);
hipError_t launch_select_keys(const Dims& dm, const float* qbar, const void* k_cache, const int32_t* kv_lens,
                              const int32_t* budgets, float* scores, int32_t* k_idx, int32_t* k_cnt, uint32_t* ws,
                              hipStream_t st, bool ws_is_zero = false);

// --- attention (attn_mfma.hip for bf16, attn_f32.hip for float32) ---------------------------------
// Cache rows attended: sparse (k_idx != nullptr): k_idx[b,kv,0..k_cnt[b,kv]); dense: 0..kv_lens[b].
struct AttnArgs {
  const void *q, *k_cache, *v_cache, *k_chunk, *v_chunk;
  const int32_t* k_idx;    // nullptr for dense
  const int32_t* n_cache;  // k_cnt [b,n_kv] (sparse) or kv_lens [b] (dense)
  void* out;
  float* lse;              // may be nullptr
  int adjacent = 0;        // set by the launcher: row-block assignment of the bf16 kernel (paired or adjacent)
};
hipError_t launch_attn_bf16(const Dims& dm, const AttnArgs& a, hipStream_t st);
// decode-sized chunks (g * C <= 32 query rows per KV head): split-KV kernel + merge, partials in `part`
bool attn_decode_applies(const Dims& dm);
size_t attn_decode_ws_floats(const Dims& dm);
hipError_t launch_attn_decode_bf16(const Dims& dm, const AttnArgs& a, float* part, hipStream_t st);
hipError_t launch_attn_f32(const Dims& dm, const AttnArgs& a, hipStream_t st);

// --- measurement aids (probes.hip) ------------------------------------------------------------------
hipError_t launch_probe_mfma(int blocks, int iters, float* sink, hipStream_t st);
hipError_t launch_probe_attn_mix(int blocks, int steps, float* sink, hipStream_t st);
hipError_t launch_probe_read(const void* src, size_t bytes, float* sink, hipStream_t st);

}  // namespace quoka
