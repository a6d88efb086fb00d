/*
 * libquoka -- QuoKA's per-chunk sparse attention path for one AMD MI355X (gfx950).
 *
 * Method: "QuoKA: Query-oriented KV selection for efficient LLM prefill"
 * (arXiv 2602.08722).  For one prefill chunk the library
 *   1. keeps, per query head, the N_Q chunk queries with the lowest cosine similarity
 *      to the chunk's mean query                         (Alg. 1, query sub-selection; Sec. 3.1),
 *   2. scores every cached key by the maximum over retained queries of the group-averaged
 *      query/key cosine                                   (Alg. 1, pre-aggregation; Sec. 3.2-3.3),
 *   3. keeps the B_SA best keys per KV head               (Alg. 1, topk step; Eq. 3),
 *   4. attends the chunk over [gathered keys | chunk keys] with a causal mask inside the chunk
 *                                                         (Alg. 2, attention step; Eq. 2-3).
 * A dense chunked-prefill attention (Eq. 2) is provided as the baseline.
 *
 * Conventions that hold for every entry point
 *   - `shape` is a host pointer, read during the call, never retained.
 *   - Every other pointer is a DEVICE pointer borrowed for the call; the caller owns all memory,
 *     including the workspace.  The library never allocates, frees or keeps pointers.
 *   - Tensors have head_dim contiguous; the three strides (batch, head, token) are in ELEMENTS and
 *     must be multiples of 8 (16-byte rows for bf16); base pointers must be 16-byte aligned.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null stream).
 *     No call synchronises the host: QUOKA_OK means "validated and enqueued".
 *   - Argument problems are reported before anything is launched:
 *       QUOKA_EINVAL       null pointer, non-positive size, n_q_heads % n_kv_heads != 0, bad stride, unknown flag
 *       QUOKA_EUNSUPPORTED head_dim not in {64,128}, unknown dtype, size beyond a stated limit
 *       QUOKA_EWORKSPACE   workspace smaller than quoka_workspace_bytes() says (or misaligned)
 *       QUOKA_EHIP         the HIP runtime refused a launch
 *   - Limits: n_retain <= 128, chunk_len <= 8192, max_kv_len < 2^24, max_budget <= max_kv_len,
 *     n_q_heads / n_kv_heads <= 16; the rows of one (batch, KV head) slice span less than 4 GiB
 *     (max_kv_len * kv_stride[2] * element size < 2^32, likewise chunk_len * ck_stride[2]).
 *   - kv_lens[b] == 0 is legal (first chunk): nothing is selected and attention is plain causal
 *     attention over the chunk.  A budget >= kv_lens[b] selects the whole cache.
 *   - Inputs are assumed finite (no NaN/Inf).
 *   - Calls are thread-safe for distinct streams with distinct workspaces and outputs.
 */
#ifndef QUOKA_H
#define QUOKA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  QUOKA_OK = 0,
  QUOKA_EINVAL = 1,
  QUOKA_EUNSUPPORTED = 2,
  QUOKA_EWORKSPACE = 3,
  QUOKA_EHIP = 4
} quoka_status;

typedef enum { QUOKA_F32 = 0, QUOKA_BF16 = 1 } quoka_dtype;

/* Ablation scorers (Sec. 3.2-3.3 and the appendix tables on scoring and aggregation); 0 is the method itself.
 * They change quoka_select_queries' qbar and quoka_score_keys' scores only; the query sub-selection is the same. */
enum {
  QUOKA_SCORE_DOT = 1,  /* dot products instead of cosines: neither the retained queries nor the keys are normalised */
  QUOKA_SCORE_MEAN = 2, /* mean instead of max over the retained-query axis                                          */
  QUOKA_SCORE_QBAR_BF16 = 8, /* cheaper Qbar K^T (the direction the paper's conclusion names): Qbar is rounded to
                                bfloat16 (nearest, ties to even) before the product; scores then differ from the
                                exact ones by at most 2^-9 * sum_i |qbar_i| (times ||k|| with QUOKA_SCORE_DOT)     */
  QUOKA_SELECT_UNIFORM = 4, /* uniformly sampled queries (the query-sampling baseline of Sec. 4) instead of the lowest
                               cosines: positions floor(r * C / N_Q), r = 0..N_Q-1, the same for every head          */
  QUOKA_ATTN_SCALE_F32 = 16 /* attention (quoka_sparse_attn, quoka_dense_attn and the calls built on them), bfloat16
                               prefill-sized chunks: apply the 1/sqrt(d) of Eq. 2-3 to the float32 products Q K^T.
                               Without the flag the factor is multiplied into the bfloat16 Q operand, which saves a
                               vector instruction per score (the kernel is 4-9 % faster) and rounds Q once more: the
                               logits then carry a relative error of 2^-9, invisible for unit-variance inputs (output
                               error 0.001 either way) and growing with the size of the logits -- 0.03 absolute in the
                               output at four times that size, 0.06 at eight, where the flag keeps it at 0.015.  Other
                               kernels (float32, decode-sized chunks) always scale in float32                       */
};

/* Problem description.  Notation of the paper: b, n_Q, n_KV, d, B_CP (chunk_len), T (kv length),
 * N_Q (n_retain), B_SA (budget). */
typedef struct quoka_shape {
  int32_t batch;        /* b                                                                  */
  int32_t n_q_heads;    /* n_Q; q-head h uses KV head h / (n_Q / n_KV)                        */
  int32_t n_kv_heads;   /* n_KV                                                               */
  int32_t head_dim;     /* d: 64 or 128                                                       */
  int32_t chunk_len;    /* C = B_CP, the same for every sequence of the batch                 */
  int32_t max_kv_len;   /* T_max: extent of the cache's token axis (may be 0)                 */
  int32_t n_retain;     /* N_Q; N' = min(N_Q, C) queries are retained                         */
  int32_t max_budget;   /* B_max: extent of k_idx's last axis                                 */
  int32_t dtype;        /* quoka_dtype of Q, K, V, chunk K/V and O                            */
  int32_t score_flags;  /* 0, or an OR of the QUOKA_SCORE_* / QUOKA_SELECT_* flags above                 */
  int64_t q_stride[3];  /* Q        [b, n_Q,  C,     d]: batch, head, token strides (elements) */
  int64_t kv_stride[3]; /* K, V     [b, n_KV, T_max, d] (K and V share strides)               */
  int64_t ck_stride[3]; /* chunk KV [b, n_KV, C,     d] (chunk K and V share strides)         */
  int64_t o_stride[3];  /* O        [b, n_Q,  C,     d]                                       */
} quoka_shape;

/* Bytes of device workspace that any entry point below may need for `shape`
 * (one number covers all of them; the buffer must be 256-byte aligned). */
quoka_status quoka_workspace_bytes(const quoka_shape* shape, size_t* out_bytes);

/* Query sub-selection and pre-aggregation (Alg. 1: mean, CosSim, topk(-S_Q, N_Q), normalise,
 * group mean; Sec. 3.1 and 3.3).
 *   q      in   [b, n_Q, C, d] (shape.dtype)
 *   q_idx  out  [b, n_Q, N'] int32: retained chunk positions per q-head, ordered by ascending
 *               cosine to the head's mean query (ties: lower position first); 0..C-1 if C <= N_Q;
 *               with QUOKA_SELECT_UNIFORM (and C > N_Q) the positions floor(r * C / N_Q) in ascending order
 *   qbar   out  [b, n_KV, N', d] float32, dense: row r = mean over the heads of the KV group of the
 *               unit-normalised r-th retained query (norms clamped at 1e-8; not re-normalised);
 *               with QUOKA_SCORE_DOT the retained queries are averaged as they are              */
quoka_status quoka_select_queries(const quoka_shape* shape, const void* q, int32_t* q_idx, float* qbar,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* Key scoring (Alg. 1: K normalisation, S = Qbar K^T, max over the query axis; Sec. 3.2-3.3).
 *   qbar     in   [b, n_KV, N', d] float32 (as written by quoka_select_queries)
 *   k_cache  in   [b, n_KV, T_max, d] (shape.dtype)
 *   kv_lens  in   [b] int32, 0 <= kv_lens[b] <= T_max
 *   scores   out  [b, n_KV, T_max] float32: scores[b,kv,t] = max_r <qbar[b,kv,r], K[b,kv,t]> /
 *                 max(||K[b,kv,t]||, 1e-8) for t < kv_lens[b]; entries t >= kv_lens[b] unspecified.
 *                 QUOKA_SCORE_DOT drops the division, QUOKA_SCORE_MEAN replaces max_r by the mean over r.
 * The product is accumulated in float32; for bf16 keys Qbar enters as an exact three-term bf16 split
 * (one term, Qbar rounded to bf16, with QUOKA_SCORE_QBAR_BF16). */
quoka_status quoka_score_keys(const quoka_shape* shape, const float* qbar, const void* k_cache,
                              const int32_t* kv_lens, float* scores, void* workspace, size_t workspace_bytes,
                              void* stream);

/* Key selection (Alg. 1: I = topk(S-hat, B_SA); Eq. 3).
 *   scores   in   [b, n_KV, T_max] float32
 *   kv_lens  in   [b] int32;  budgets in [b] int32 (B_SA per sequence, >= 0)
 *   k_idx    out  [b, n_KV, B_max] int32: the k_cnt best positions, ASCENDING; equal scores go to the
 *                 lower position; entries past k_cnt unspecified
 *   k_cnt    out  [b, n_KV] int32 = min(budgets[b], kv_lens[b], B_max)                             */
quoka_status quoka_topk_keys(const quoka_shape* shape, const float* scores, const int32_t* kv_lens,
                             const int32_t* budgets, int32_t* k_idx, int32_t* k_cnt, void* workspace,
                             size_t workspace_bytes, void* stream);

/* Key scoring and key selection as one stage (Alg. 1: S = Qbar K^T, S-hat = max, I = topk(S-hat, B_SA); the
 * conclusion's "more efficient Qbar K^T").  Arguments as in quoka_score_keys and quoka_topk_keys.
 *   k_idx, k_cnt  out  exactly what quoka_score_keys followed by quoka_topk_keys writes: the top-B of the exact
 *                      scores, equal scores to the lower position, ascending.
 *   scores        out  [b, n_KV, T_max] float32.  For bf16 caches longer than 32768 positions scored with the method's
 *                      own rule (no QUOKA_SCORE_* flag) the stage scores every key with a single bf16 term of Qbar
 *                      first and repeats the exact three-term product only for the keys whose provisional score lies
 *                      within the proven error bound of the provisional cut; `scores` then holds the exact value
 *                      (as quoka_score_keys computes it, bit for bit) for those keys -- at least every key within
 *                      2^-11 of the cut -- and elsewhere the provisional value, which differs from the exact one by at
 *                      most max_r ||qbar_r - bf16(qbar_r)||_2 + 4e-6 (<= 2^-9).  In every other case the stage is the
 *                      two separate calls and `scores` is exact everywhere.                                          */
quoka_status quoka_select_keys(const quoka_shape* shape, const float* qbar, const void* k_cache,
                               const int32_t* kv_lens, const int32_t* budgets, float* scores, int32_t* k_idx,
                               int32_t* k_cnt, void* workspace, size_t workspace_bytes, void* stream);

/* Chunk attention over the gathered cache rows and the chunk's own keys/values (Alg. 2 attention
 * step; Eq. 2-3).  For q-head h (KV head kv), chunk position i:
 *   O[b,h,i] = sum_j softmax_j(<Q[b,h,i], K_j> / sqrt(d)) V_j,
 *   j over cache rows k_idx[b,kv,0..k_cnt[b,kv]) and chunk rows c <= i.
 *   q, k_cache, v_cache, k_chunk, v_chunk  in (shape.dtype);  out [b, n_Q, C, d] (shape.dtype)
 *   k_idx [b, n_KV, B_max], k_cnt [b, n_KV] as written by quoka_topk_keys (any order is accepted;
 *   every index must be in [0, T_max): the kernels clamp an index outside that range to row T_max - 1,
 *   so a malformed list gives a wrong result but never an access outside the cache)
 *   lse   out, optional (may be NULL) [b, n_Q, C] float32: natural-log softmax normaliser per row.
 * bf16: QK^T and PV run on bf16 MFMA with float32 accumulation and float32 softmax state; the
 *   factor log2(e)/sqrt(d) is multiplied into Q beforehand and P is the MFMA operand, so Q and P are
 *   each rounded to bf16 once (outputs agree with exact arithmetic on the bf16 inputs to about 1e-2);
 * f32: all arithmetic in float32.                                                                  */
quoka_status quoka_sparse_attn(const quoka_shape* shape, const void* q, const void* k_cache, const void* v_cache,
                               const int32_t* k_idx, const int32_t* k_cnt, const void* k_chunk,
                               const void* v_chunk, void* out, float* lse, void* workspace,
                               size_t workspace_bytes, void* stream);

/* Dense chunked-prefill attention, the baseline (Eq. 2): as quoka_sparse_attn with j over all cache
 * rows t < kv_lens[b] and chunk rows c <= i. */
quoka_status quoka_dense_attn(const quoka_shape* shape, const void* q, const void* k_cache, const void* v_cache,
                              const int32_t* kv_lens, const void* k_chunk, const void* v_chunk, void* out,
                              float* lse, void* workspace, size_t workspace_bytes, void* stream);

/* The sparse stages back to back on one stream (Alg. 2, select-then-attend for one chunk): quoka_select_queries,
 * quoka_select_keys, quoka_sparse_attn.  Intermediates are returned to the caller: q_idx, qbar, k_idx, k_cnt as
 * above, scores as quoka_select_keys leaves them. */
quoka_status quoka_chunk_attn(const quoka_shape* shape, const void* q, const void* k_cache, const void* v_cache,
                              const int32_t* kv_lens, const int32_t* budgets, const void* k_chunk,
                              const void* v_chunk, int32_t* q_idx, float* qbar, float* scores, int32_t* k_idx,
                              int32_t* k_cnt, void* out, float* lse, void* workspace, size_t workspace_bytes,
                              void* stream);

/* Chunked prefill of a whole prompt, one layer (Alg. 2: for every chunk select, attend, then append the chunk to
 * the cache).  K and V hold the whole prompt, so the chunk's keys and values already sit behind the cache rows and
 * the append step is the cache length moving forward by one chunk: nothing is copied.
 *   shape     chunk_len = B_CP; max_kv_len = L, the prompt length (extent of the token axis of q, k, v and out);
 *             kv_stride describes K and V [b, n_KV, L, d]; ck_stride is ignored (chunk rows are rows of K and V);
 *             q_stride / o_stride describe Q and O [b, n_Q, L, d].  All sequences of the batch have length L.
 *   q, k, v   in  (shape.dtype);  out  [b, n_Q, L, d] (shape.dtype)
 *   kv_lens_all  in  [n_chunks, b] int32, n_chunks = ceil(L / chunk_len): the cache length before chunk i, i.e.
 *                i * chunk_len in every entry (a device array because every stage reads its lengths from memory)
 *   budgets_all  in  [n_chunks, b] int32: B_SA for chunk i (ignored when sparse == 0)
 *   sparse    non-zero: quoka_chunk_attn per chunk; zero: quoka_dense_attn per chunk (the baseline of Eq. 2, which
 *             over a whole prompt equals plain causal attention)
 *   q_idx, qbar, scores, k_idx, k_cnt   scratch for one chunk, shaped as in quoka_chunk_attn; they hold the last
 *             chunk's intermediates on return (unused when sparse == 0, may then be NULL)
 * The last chunk may be shorter than chunk_len.  Everything is enqueued on `stream`, chunk after chunk.          */
quoka_status quoka_prefill_attn(const quoka_shape* shape, int sparse, const void* q, const void* k, const void* v,
                                const int32_t* kv_lens_all, const int32_t* budgets_all, int32_t* q_idx, float* qbar,
                                float* scores, int32_t* k_idx, int32_t* k_cnt, void* out, void* workspace,
                                size_t workspace_bytes, void* stream);

/* quoka_topk_keys for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus the workspace, same
 * results bit for bit.  The histograms and per-tile counts of the multi-block path (max_kv_len > 32768) live in a
 * 4 MiB array inside the library instead (one copy per GPU, held until the process ends); the call allocates
 * nothing and frees nothing.  QUOKA_EWORKSPACE if the shape needs more than that array holds, i.e. if
 *   batch * n_kv_heads * (6152 + 2 * ceil(max_kv_len / 2048)) * 4 bytes > QUOKA_NOALLOC_SCRATCH_BYTES
 * (e.g. 64 KV-head slices of 131072 tokens need 1.6 MiB).  The call clears what it needs itself, so the array may
 * hold anything on entry.  All calls on one GPU share that GPU's array: two such calls that overlap in time on the
 * same GPU (different streams or threads) race; calls on one stream, or ordered by events, are safe.            */
#define QUOKA_NOALLOC_SCRATCH_BYTES (4u << 20)
quoka_status quoka_topk_keys_noalloc(const quoka_shape* shape, const float* scores, const int32_t* kv_lens,
                                     const int32_t* budgets, int32_t* k_idx, int32_t* k_cnt, void* stream);

/* Measurement aids (no part of the method): kernels of known work for a benchmark to time beside the library's
 * own kernels, so that rates can be quoted against what the GPU sustains as well as against its published peaks.
 *   quoka_probe_mfma  `blocks` blocks of 4 waves, each wave issuing 4 * iters register-only
 *                     v_mfma_f32_32x32x16_bf16 (32768 flop each); sink: device float, never written in practice.
 *   quoka_probe_read  reads `bytes` (multiple of 16; src 16-byte aligned, device memory) once with coalesced
 *                     16-byte loads and writes nothing.
 *   quoka_probe_attn_mix  `blocks` blocks of 8 waves, each wave running `steps` steps of the bf16 attention kernel's
 *                     instruction mix without its memory side: 32 MFMAs (32768 flop each), 32 exponentials and about
 *                     160 plain vector operations per step.  Its rate is the ceiling of that work split.        */
quoka_status quoka_probe_attn_mix(int blocks, int steps, float* sink, void* stream);
quoka_status quoka_probe_mfma(int blocks, int iters, float* sink, void* stream);
quoka_status quoka_probe_read(const void* src, size_t bytes, float* sink, void* stream);

const char* quoka_status_string(quoka_status status);

/* major * 10000 + minor * 100 + patch */
int quoka_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QUOKA_H */
