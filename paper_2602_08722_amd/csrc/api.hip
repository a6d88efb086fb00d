// C-ABI layer of libquoka: argument validation, workspace carving, kernel dispatch.
// Nothing here allocates or synchronises; the only state kept is the per-device address of the library-owned
// scratch array of quoka_topk_keys_noalloc.
#include <hip/hip_runtime.h>

#include <atomic>

#include "kernels.h"
#include "quoka.h"

namespace {

using quoka::Dims;

constexpr int kMaxRetain = 128;
constexpr int kMaxGroup = 16;   // q-heads per KV head
constexpr int kMaxChunk = 8192;
constexpr int kMaxKv = 1 << 24;
constexpr size_t kAlign = 256;

size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct WsLayout {
  size_t select_off, select_bytes;
  size_t topk_off, topk_bytes;
  size_t sel_off, sel_bytes;
  size_t decode_off, decode_bytes;
  size_t total;
};

quoka_status check_shape(const quoka_shape* s, Dims* dm) {
  if (s == nullptr) return QUOKA_EINVAL;
  if (s->batch < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->chunk_len < 1 || s->n_retain < 1 ||
      s->max_kv_len < 0 || s->max_budget < 0 || (s->score_flags & ~(QUOKA_SCORE_DOT | QUOKA_SCORE_MEAN | QUOKA_SELECT_UNIFORM | QUOKA_SCORE_QBAR_BF16 |
                          QUOKA_ATTN_SCALE_F32)) != 0)
    return QUOKA_EINVAL;
  if (s->n_q_heads % s->n_kv_heads != 0) return QUOKA_EINVAL;
  if (s->max_budget > s->max_kv_len) return QUOKA_EINVAL;
  if (s->dtype != QUOKA_F32 && s->dtype != QUOKA_BF16) return QUOKA_EUNSUPPORTED;
  if (s->head_dim != 64 && s->head_dim != 128) return QUOKA_EUNSUPPORTED;
  if (s->n_retain > kMaxRetain || s->chunk_len > kMaxChunk || s->max_kv_len >= kMaxKv) return QUOKA_EUNSUPPORTED;
  if (s->n_q_heads / s->n_kv_heads > kMaxGroup) return QUOKA_EUNSUPPORTED;
  if ((long long)s->batch * s->n_q_heads > 65535 || s->batch > 65535) return QUOKA_EUNSUPPORTED;
  const int64_t* strides[4] = {s->q_stride, s->kv_stride, s->ck_stride, s->o_stride};
  for (const int64_t* st : strides) {
    for (int i = 0; i < 3; ++i)
      if (st[i] < 0 || st[i] % 8 != 0) return QUOKA_EINVAL;
    if (st[2] < s->head_dim) return QUOKA_EINVAL;
  }
  // kernels address the rows of one (batch, KV head) slice with 32-bit byte offsets
  const int es = s->dtype == QUOKA_BF16 ? 2 : 4;
  if ((unsigned long long)s->max_kv_len * (unsigned long long)s->kv_stride[2] * es >= (1ull << 32) ||
      (unsigned long long)s->chunk_len * (unsigned long long)s->ck_stride[2] * es >= (1ull << 32))
    return QUOKA_EUNSUPPORTED;
  dm->b = s->batch;
  dm->n_q = s->n_q_heads;
  dm->n_kv = s->n_kv_heads;
  dm->g = s->n_q_heads / s->n_kv_heads;
  dm->d = s->head_dim;
  dm->C = s->chunk_len;
  dm->T_max = s->max_kv_len;
  dm->n_ret = s->n_retain;
  dm->B_max = s->max_budget;
  dm->flags = s->score_flags;
  for (int i = 0; i < 3; ++i) {
    dm->qs[i] = s->q_stride[i];
    dm->kvs[i] = s->kv_stride[i];
    dm->cks[i] = s->ck_stride[i];
    dm->os[i] = s->o_stride[i];
  }
  return QUOKA_OK;
}

WsLayout layout(const Dims& dm) {
  WsLayout l;
  l.select_off = 0;
  l.select_bytes = round_up(quoka::select_queries_ws_floats(dm) * sizeof(float), kAlign);
  l.topk_off = l.select_off + l.select_bytes;
  l.topk_bytes = round_up(quoka::topk_ws_words(dm) * sizeof(uint32_t), kAlign);
  l.sel_off = l.topk_off + l.topk_bytes;
  l.sel_bytes = round_up(quoka::select_keys_ws_words(dm) * sizeof(uint32_t), kAlign);
  l.decode_off = l.sel_off + l.sel_bytes;
  l.decode_bytes = dm.b > 0 ? round_up(quoka::attn_decode_ws_floats(dm) * sizeof(float), kAlign) : 0;
  l.total = l.decode_off + l.decode_bytes;
  if (l.total == 0) l.total = kAlign;
  return l;
}

quoka_status check_ws(const WsLayout& l, const void* ws, size_t bytes) {
  if (ws == nullptr) return QUOKA_EINVAL;
  if (reinterpret_cast<uintptr_t>(ws) % kAlign != 0) return QUOKA_EWORKSPACE;
  if (bytes < l.total) return QUOKA_EWORKSPACE;
  return QUOKA_OK;
}

bool aligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

quoka_status from_hip(hipError_t e) { return e == hipSuccess ? QUOKA_OK : QUOKA_EHIP; }

}  // namespace

// ---- entry point for callers that cannot allocate ------------------------------------------------------------
// The multi-block top-k's histograms, cut steps and per-tile counts in an array the library owns.  `scratch` is the
// host-side handle of the device array; its device address differs per GPU and is looked up once per device with
// that device current.  Host code below only ever uses the looked-up pointer.
namespace {
constexpr size_t kScratchWords = QUOKA_NOALLOC_SCRATCH_BYTES / sizeof(uint32_t);
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) uint32_t scratch[kScratchWords];
static std::atomic<uint32_t*> g_scratch_ptr[kMaxDevices];

static hipError_t scratch_address(uint32_t** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  uint32_t* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    void* sym = nullptr;
    e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));   // this device's copy of the array
    if (e != hipSuccess) return e;
    if (sym == nullptr) return hipErrorInvalidSymbol;
    p = static_cast<uint32_t*>(sym);
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // (two threads racing here store the same address)
  }
  *out = p;
  return hipSuccess;
}

extern "C" {

quoka_status quoka_workspace_bytes(const quoka_shape* shape, size_t* out_bytes) {
  Dims dm;
  quoka_status st = check_shape(shape, &dm);
  if (st != QUOKA_OK) return st;
  if (out_bytes == nullptr) return QUOKA_EINVAL;
  *out_bytes = layout(dm).total;
  return QUOKA_OK;
}

quoka_status quoka_select_queries(const quoka_shape* shape, const void* q, int32_t* q_idx, float* qbar,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  Dims dm;
  quoka_status st = check_shape(shape, &dm);
  if (st != QUOKA_OK) return st;
  if (q == nullptr || q_idx == nullptr || qbar == nullptr) return QUOKA_EINVAL;
  if (!aligned16(q) || !aligned16(qbar)) return QUOKA_EINVAL;
  const WsLayout l = layout(dm);
  st = check_ws(l, workspace, workspace_bytes);
  if (st != QUOKA_OK) return st;
  float* ws = reinterpret_cast<float*>(static_cast<char*>(workspace) + l.select_off);
  return from_hip(quoka::launch_select_queries(dm, shape->dtype, q, q_idx, qbar, ws, static_cast<hipStream_t>(stream)));
}

quoka_status quoka_score_keys(const quoka_shape* shape, const float* qbar, const void* k_cache,
                              const int32_t* kv_lens, float* scores, void* workspace, size_t workspace_bytes,
                              void* stream) {
  Dims dm;
  quoka_status st = check_shape(shape, &dm);
  if (st != QUOKA_OK) return st;
  if (qbar == nullptr || kv_lens == nullptr) return QUOKA_EINVAL;
  if (dm.T_max > 0 && (k_cache == nullptr || scores == nullptr)) return QUOKA_EINVAL;
  if (!aligned16(qbar) || !aligned16(k_cache)) return QUOKA_EINVAL;
  st = check_ws(layout(dm), workspace, workspace_bytes);
  if (st != QUOKA_OK) return st;
  return from_hip(
      quoka::launch_score_keys(dm, shape->dtype, qbar, k_cache, kv_lens, scores, static_cast<hipStream_t>(stream)));
}

quoka_status quoka_topk_keys(const quoka_shape* shape, const float* scores, const int32_t* kv_lens,
                             const int32_t* budgets, int32_t* k_idx, int32_t* k_cnt, void* workspace,
                             size_t workspace_bytes, void* stream) {
  Dims dm;
  quoka_status st = check_shape(shape, &dm);
  if (st != QUOKA_OK) return st;
  if (kv_lens == nullptr || budgets == nullptr || k_cnt == nullptr) return QUOKA_EINVAL;
  if (dm.T_max > 0 && scores == nullptr) return QUOKA_EINVAL;
  if (dm.B_max > 0 && k_idx == nullptr) return QUOKA_EINVAL;
  const WsLayout l = layout(dm);
  st = check_ws(l, workspace, workspace_bytes);
  if (st != QUOKA_OK) return st;
  uint32_t* ws = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + l.topk_off);
  return from_hip(
      quoka::launch_topk_keys(dm, scores, kv_lens, budgets, k_idx, k_cnt, ws, static_cast<hipStream_t>(stream)));
}

static quoka_status attn_common(const quoka_shape* shape, const void* q, const void* k_cache, const void* v_cache,
                                const int32_t* k_idx, const int32_t* n_cache, bool sparse, const void* k_chunk,
                                const void* v_chunk, void* out, float* lse, void* workspace, size_t workspace_bytes,
                                void* stream) {
  Dims dm;
  quoka_status st = check_shape(shape, &dm);
  if (st != QUOKA_OK) return st;
  if (q == nullptr || k_chunk == nullptr || v_chunk == nullptr || out == nullptr || n_cache == nullptr)
    return QUOKA_EINVAL;
  const bool has_cache = sparse ? dm.B_max > 0 : dm.T_max > 0;
  if (has_cache && (k_cache == nullptr || v_cache == nullptr)) return QUOKA_EINVAL;
  if (sparse && dm.B_max > 0 && k_idx == nullptr) return QUOKA_EINVAL;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(k_chunk) || !aligned16(v_chunk) ||
      !aligned16(out))
    return QUOKA_EINVAL;
  const WsLayout l = layout(dm);
  st = check_ws(l, workspace, workspace_bytes);
  if (st != QUOKA_OK) return st;
  quoka::AttnArgs a;
  a.q = q;
  a.k_cache = k_cache;
  a.v_cache = v_cache;
  a.k_chunk = k_chunk;
  a.v_chunk = v_chunk;
  // a null k_idx selects the dense kernel path, so a sparse call with B_max == 0 still needs a non-null marker:
  // n_cache is then 0 everywhere and k_idx is never dereferenced.
  a.k_idx = sparse ? (k_idx != nullptr ? k_idx : n_cache) : nullptr;
  a.n_cache = n_cache;
  a.out = out;
  a.lse = lse;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (shape->dtype == QUOKA_BF16 && quoka::attn_decode_applies(dm)) {
    float* part = reinterpret_cast<float*>(static_cast<char*>(workspace) + l.decode_off);
    return from_hip(quoka::launch_attn_decode_bf16(dm, a, part, hs));
  }
  return from_hip(shape->dtype == QUOKA_BF16 ? quoka::launch_attn_bf16(dm, a, hs) : quoka::launch_attn_f32(dm, a, hs));
}

quoka_status quoka_sparse_attn(const quoka_shape* shape, const void* q, const void* k_cache, const void* v_cache,
                               const int32_t* k_idx, const int32_t* k_cnt, const void* k_chunk,
                               const void* v_chunk, void* out, float* lse, void* workspace,
                               size_t workspace_bytes, void* stream) {
  return attn_common(shape, q, k_cache, v_cache, k_idx, k_cnt, true, k_chunk, v_chunk, out, lse, workspace,
                     workspace_bytes, stream);
}

quoka_status quoka_dense_attn(const quoka_shape* shape, const void* q, const void* k_cache, const void* v_cache,
                              const int32_t* kv_lens, const void* k_chunk, const void* v_chunk, void* out,
                              float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  return attn_common(shape, q, k_cache, v_cache, nullptr, kv_lens, false, k_chunk, v_chunk, out, lse, workspace,
                     workspace_bytes, stream);
}

// Scoring and top-B of one chunk on `stream`: the two-pass stage where it applies, else the two separate launches
// (whose scoring launch clears the multi-block top-k's histograms).
static quoka_status select_keys_common(const Dims& dm, int dtype, const float* qbar, const void* k_cache,
                                       const int32_t* kv_lens, const int32_t* budgets, float* scores, int32_t* k_idx,
                                       int32_t* k_cnt, void* workspace, const WsLayout& l, hipStream_t hs,
                                       bool sel_ws_is_zero) {
  if (dm.T_max > 0 && quoka::select_keys_two_pass_applies(dm, dtype)) {
    uint32_t* sel_ws = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + l.sel_off);
    return from_hip(quoka::launch_select_keys(dm, qbar, k_cache, kv_lens, budgets, scores, k_idx, k_cnt, sel_ws, hs,
                                              sel_ws_is_zero));
  }
  uint32_t* topk_ws = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + l.topk_off);
  const size_t topk_words = quoka::topk_ws_words(dm);
  const bool fuse_clear = dm.T_max > 0 && topk_words > 0;
  quoka_status st = from_hip(quoka::launch_score_keys(dm, dtype, qbar, k_cache, kv_lens, scores, hs,
                                                      fuse_clear ? topk_ws : nullptr, fuse_clear ? topk_words : 0));
  if (st != QUOKA_OK) return st;
  return from_hip(quoka::launch_topk_keys(dm, scores, kv_lens, budgets, k_idx, k_cnt, topk_ws, hs, fuse_clear));
}

quoka_status quoka_select_keys(const quoka_shape* shape, const float* qbar, const void* k_cache,
                               const int32_t* kv_lens, const int32_t* budgets, float* scores, int32_t* k_idx,
                               int32_t* k_cnt, void* workspace, size_t workspace_bytes, void* stream) {
  Dims dm;
  quoka_status st = check_shape(shape, &dm);
  if (st != QUOKA_OK) return st;
  if (qbar == nullptr || kv_lens == nullptr || budgets == nullptr || k_cnt == nullptr) return QUOKA_EINVAL;
  if (dm.T_max > 0 && (k_cache == nullptr || scores == nullptr)) return QUOKA_EINVAL;
  if (dm.B_max > 0 && k_idx == nullptr) return QUOKA_EINVAL;
  if (!aligned16(qbar) || !aligned16(k_cache)) return QUOKA_EINVAL;
  const WsLayout l = layout(dm);
  st = check_ws(l, workspace, workspace_bytes);
  if (st != QUOKA_OK) return st;
  return select_keys_common(dm, shape->dtype, qbar, k_cache, kv_lens, budgets, scores, k_idx, k_cnt, workspace, l,
                            static_cast<hipStream_t>(stream), false);
}

quoka_status quoka_chunk_attn(const quoka_shape* shape, const void* q, const void* k_cache, const void* v_cache,
                              const int32_t* kv_lens, const int32_t* budgets, const void* k_chunk,
                              const void* v_chunk, int32_t* q_idx, float* qbar, float* scores, int32_t* k_idx,
                              int32_t* k_cnt, void* out, float* lse, void* workspace, size_t workspace_bytes,
                              void* stream) {
  // The stages as in quoka_select_queries / quoka_select_keys (same checks), except that the last launch of the query
  // stage also clears the histograms and counters of the two-pass key selection, which saves that stage a launch.
  Dims dm;
  quoka_status st = check_shape(shape, &dm);
  if (st != QUOKA_OK) return st;
  if (q == nullptr || q_idx == nullptr || qbar == nullptr) return QUOKA_EINVAL;
  if (kv_lens == nullptr || budgets == nullptr || k_cnt == nullptr) return QUOKA_EINVAL;
  if (dm.T_max > 0 && (k_cache == nullptr || scores == nullptr)) return QUOKA_EINVAL;
  if (dm.B_max > 0 && k_idx == nullptr) return QUOKA_EINVAL;
  if (!aligned16(q) || !aligned16(qbar) || !aligned16(k_cache)) return QUOKA_EINVAL;
  const WsLayout l = layout(dm);
  st = check_ws(l, workspace, workspace_bytes);
  if (st != QUOKA_OK) return st;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const bool two_pass = dm.T_max > 0 && quoka::select_keys_two_pass_applies(dm, shape->dtype);
  uint32_t* sel_ws = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + l.sel_off);
  float* sq_ws = reinterpret_cast<float*>(static_cast<char*>(workspace) + l.select_off);
  st = from_hip(quoka::launch_select_queries(dm, shape->dtype, q, q_idx, qbar, sq_ws, hs, two_pass ? sel_ws : nullptr,
                                             two_pass ? quoka::select_keys_zero_words(dm) : 0));
  if (st != QUOKA_OK) return st;
  st = select_keys_common(dm, shape->dtype, qbar, k_cache, kv_lens, budgets, scores, k_idx, k_cnt, workspace, l, hs,
                          two_pass);
  if (st != QUOKA_OK) return st;
  return quoka_sparse_attn(shape, q, k_cache, v_cache, k_idx, k_cnt, k_chunk, v_chunk, out, lse, workspace,
                           workspace_bytes, stream);
}

quoka_status quoka_prefill_attn(const quoka_shape* shape, int sparse, const void* q, const void* k, const void* v,
                                const int32_t* kv_lens_all, const int32_t* budgets_all, int32_t* q_idx, float* qbar,
                                float* scores, int32_t* k_idx, int32_t* k_cnt, void* out, void* workspace,
                                size_t workspace_bytes, void* stream) {
  Dims dm;
  quoka_status st = check_shape(shape, &dm);
  if (st != QUOKA_OK) return st;
  if (q == nullptr || k == nullptr || v == nullptr || out == nullptr || kv_lens_all == nullptr) return QUOKA_EINVAL;
  if (sparse && budgets_all == nullptr) return QUOKA_EINVAL;
  const int L = shape->max_kv_len, C = shape->chunk_len;
  if (L < 1) return QUOKA_EINVAL;
  const size_t es = shape->dtype == QUOKA_BF16 ? 2 : 4;
  const int n_chunks = (L + C - 1) / C;
  for (int i = 0; i < n_chunks; ++i) {
    quoka_shape sh = *shape;
    sh.chunk_len = (i + 1) * C <= L ? C : L - i * C;   // the last chunk may be short
    for (int a = 0; a < 3; ++a) sh.ck_stride[a] = shape->kv_stride[a];
    const size_t tok = (size_t)i * C;
    const char* qi = static_cast<const char*>(q) + tok * shape->q_stride[2] * es;
    const char* ki = static_cast<const char*>(k) + tok * shape->kv_stride[2] * es;
    const char* vi = static_cast<const char*>(v) + tok * shape->kv_stride[2] * es;
    char* oi = static_cast<char*>(out) + tok * shape->o_stride[2] * es;
    const int32_t* lens = kv_lens_all + (size_t)i * shape->batch;
    if (sparse) {
      st = quoka_chunk_attn(&sh, qi, k, v, lens, budgets_all + (size_t)i * shape->batch, ki, vi, q_idx, qbar, scores,
                            k_idx, k_cnt, oi, nullptr, workspace, workspace_bytes, stream);
    } else {
      st = quoka_dense_attn(&sh, qi, k, v, lens, ki, vi, oi, nullptr, workspace, workspace_bytes, stream);
    }
    if (st != QUOKA_OK) return st;
  }
  return QUOKA_OK;
}

quoka_status quoka_topk_keys_noalloc(const quoka_shape* shape, const float* scores, const int32_t* kv_lens,
                                     const int32_t* budgets, int32_t* k_idx, int32_t* k_cnt, void* stream) {
  Dims dm;
  quoka_status st = check_shape(shape, &dm);
  if (st != QUOKA_OK) return st;
  if (kv_lens == nullptr || budgets == nullptr || k_cnt == nullptr) return QUOKA_EINVAL;
  if (dm.T_max > 0 && scores == nullptr) return QUOKA_EINVAL;
  if (dm.B_max > 0 && k_idx == nullptr) return QUOKA_EINVAL;
  if (quoka::topk_ws_words(dm) > kScratchWords) return QUOKA_EWORKSPACE;
  uint32_t* ws = nullptr;
  if (scratch_address(&ws) != hipSuccess) return QUOKA_EHIP;
  // the launcher clears the words it uses with a fill kernel of its own (no memset node, nothing allocated)
  return from_hip(
      quoka::launch_topk_keys(dm, scores, kv_lens, budgets, k_idx, k_cnt, ws, static_cast<hipStream_t>(stream)));
}

quoka_status quoka_probe_mfma(int blocks, int iters, float* sink, void* stream) {
  if (blocks < 1 || blocks > 65535 || iters < 1 || sink == nullptr) return QUOKA_EINVAL;
  return from_hip(quoka::launch_probe_mfma(blocks, iters, sink, static_cast<hipStream_t>(stream)));
}

quoka_status quoka_probe_attn_mix(int blocks, int steps, float* sink, void* stream) {
  if (blocks < 1 || blocks > 65535 || steps < 1 || sink == nullptr) return QUOKA_EINVAL;
  return from_hip(quoka::launch_probe_attn_mix(blocks, steps, sink, static_cast<hipStream_t>(stream)));
}

quoka_status quoka_probe_read(const void* src, size_t bytes, float* sink, void* stream) {
  if (src == nullptr || sink == nullptr || bytes == 0 || bytes % 16 != 0 || !aligned16(src)) return QUOKA_EINVAL;
  return from_hip(quoka::launch_probe_read(src, bytes, sink, static_cast<hipStream_t>(stream)));
}

const char* quoka_status_string(quoka_status status) {
  switch (status) {
    case QUOKA_OK: return "ok";
    case QUOKA_EINVAL: return "invalid argument";
    case QUOKA_EUNSUPPORTED: return "unsupported shape or dtype";
    case QUOKA_EWORKSPACE: return "workspace too small or misaligned";
    case QUOKA_EHIP: return "HIP launch failed";
  }
  return "unknown status";
}

int quoka_version(void) { return 100; }

}  // extern "C"
