"""CPU oracle for QuoKA's per-chunk attention path -- TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 numpy transcription of the method as the paper states it
(Algorithm 1: KV sub-selection; Algorithm 2, the two lines that select and then
attend; Eq. 1-3: attention, chunked prefill, gather).  It exists to check the HIP
library against and must never be on the product path: only tests, the smoke
check and the benchmark's cpu_baseline leg may import it.  It shares no code
with the HIP path and imports nothing from it.

Everything works on ONE sequence (no batch axis); callers loop over sequences.
Shapes:  Q [n_q, C, d]   K, V [n_kv, T, d]   Kc, Vc [n_kv, C, d].

Readings taken where the paper is silent (each is listed with its reason in the
design notes of the repository):
  * retained queries are kept in rank order (ascending cosine to the mean query),
    ties broken by the lower token index;
  * key/query normalisation is used for scoring only -- attention runs on the
    original K, V and on all C chunk queries (Alg. 2 attends with Q_i itself);
  * selection ranges over the past cache only; the chunk's own keys are always
    attended, causally, diagonal included;
  * the group mean of unit queries is not re-normalised (needed for the
    pre-aggregation identity of Sec. 3.3);
  * q-head h belongs to KV head h // (n_q / n_kv);
  * norms are clamped from below at EPS; top-k ties go to the lower index;
  * selected key indices are reported in ascending position.

Pins: see tests/test_oracle_*.py.  Unpinned by the paper (no worked example is
printed): the rank-order and tie-break conventions above -- "parity unpinned"
for those two readings; everything else is pinned by invariants, closed forms,
brute force and library routines.
"""
from __future__ import annotations

import numpy as np

EPS = 1e-8


# ---------------------------------------------------------------------------
# Alg. 1, query sub-selection block
# ---------------------------------------------------------------------------
def mean_query(Q: np.ndarray) -> np.ndarray:
    """M_Q = mean over the chunk's tokens, one per q-head (Alg. 1, mean step)."""
    Q = np.asarray(Q, dtype=np.float64)
    return Q.mean(axis=1)


def cos_to_mean(Q: np.ndarray) -> np.ndarray:
    """S_Q[h, i] = CosSim(Q[h, i], M_Q[h]) (Alg. 1, CosSim step; Sec. 3.1)."""
    Q = np.asarray(Q, dtype=np.float64)
    M = mean_query(Q)
    dots = np.einsum("hcd,hd->hc", Q, M)
    qn = np.maximum(np.sqrt(np.einsum("hcd,hcd->hc", Q, Q)), EPS)
    mn = np.maximum(np.sqrt(np.einsum("hd,hd->h", M, M)), EPS)
    return dots / (qn * mn[:, None])


def select_queries(Q: np.ndarray, n_retain: int, rule: str = "cosine") -> np.ndarray:
    """Indices of the retained queries per q-head.

    Alg. 1: only when the chunk is longer than N_Q, keep the N_Q queries that
    rank highest by -CosSim(M_Q, q), i.e. the lowest cosines, in rank order;
    otherwise keep all queries in position order.

    rule="uniform" is the query-sampling baseline the experiments compare with
    (Sec. 4, sparse attention baselines: queries sampled uniformly): the N_Q
    positions floor(r * C / N_Q), r = 0..N_Q-1, the same for every head.  The
    paper does not say how the uniform sample is drawn; an even stride is the
    deterministic form of it (reading listed in the design notes).
    """
    assert rule in ("cosine", "uniform")
    Q = np.asarray(Q, dtype=np.float64)
    n_q, C, _ = Q.shape
    if C <= n_retain:
        return np.tile(np.arange(C, dtype=np.int64), (n_q, 1))
    if rule == "uniform":
        pos = [(r * C) // n_retain for r in range(n_retain)]
        return np.tile(np.asarray(pos, dtype=np.int64), (n_q, 1))
    s = cos_to_mean(Q)
    order = np.argsort(s, axis=1, kind="stable")  # ascending cosine, ties -> lower index
    return order[:, :n_retain].astype(np.int64)


def unit(x: np.ndarray) -> np.ndarray:
    """x / max(||x||, EPS) along the last axis (Alg. 1, the two normalisation steps)."""
    x = np.asarray(x, dtype=np.float64)
    n = np.sqrt(np.sum(x * x, axis=-1, keepdims=True))
    return x / np.maximum(n, EPS)


def group_mean_queries(Q: np.ndarray, q_idx: np.ndarray, n_kv: int, similarity: str = "cosine") -> np.ndarray:
    """Q-bar [n_kv, N', d]: mean over each KV group of the unit retained queries.

    Alg. 1, pre-aggregation step: reshape (n_kv, n_q/n_kv, N_Q, d) and average
    the group axis; the r-th retained query of every head in a group is paired.
    similarity="dot" is the ablation of Sec. 3.2 (dot products instead of
    cosines): the retained queries are averaged without normalisation.
    """
    assert similarity in ("cosine", "dot")
    Q = np.asarray(Q, dtype=np.float64)
    n_q = Q.shape[0]
    g = n_q // n_kv
    Qr = np.stack([Q[h, q_idx[h]] for h in range(n_q)])  # [n_q, N', d]
    if similarity == "cosine":
        Qr = unit(Qr)
    return Qr.reshape(n_kv, g, Qr.shape[1], Qr.shape[2]).mean(axis=1)


# ---------------------------------------------------------------------------
# Alg. 1, scoring and aggregation
# ---------------------------------------------------------------------------
def key_scores(Q: np.ndarray, q_idx: np.ndarray, K: np.ndarray, n_kv: int, similarity: str = "cosine",
               reduce: str = "max") -> np.ndarray:
    """S-hat [n_kv, T], literal (post-hoc) form of Sec. 3.2-3.3.

    Per q-head cosine between every retained query and every key, averaged over
    the heads of a KV group, then the maximum over the retained-query axis.
    The two ablations of Sec. 3.2-3.3 (appendix tables on scoring and aggregation):
    similarity="dot" scores with plain dot products (no normalisation of queries
    or keys); reduce="mean" averages over the retained-query axis instead of
    taking the maximum.
    """
    assert similarity in ("cosine", "dot") and reduce in ("max", "mean")
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    n_q = Q.shape[0]
    g = n_q // n_kv
    T = K.shape[1]
    Kn = unit(K) if similarity == "cosine" else K
    out = np.empty((n_kv, T), dtype=np.float64)
    for kv in range(n_kv):
        acc = None
        for j in range(g):
            h = kv * g + j
            qn = Q[h, q_idx[h]]                  # [N', d]
            if similarity == "cosine":
                qn = unit(qn)
            S = qn @ Kn[kv].T                    # cosines (or dot products) [N', T]
            acc = S if acc is None else acc + S
        if T == 0:
            out[kv] = np.empty((0,))
        else:
            out[kv] = (acc / g).max(axis=0) if reduce == "max" else (acc / g).mean(axis=0)
    return out


def key_scores_preagg(qbar: np.ndarray, K: np.ndarray, similarity: str = "cosine", reduce: str = "max") -> np.ndarray:
    """S-hat [n_kv, T] from a given Q-bar: max_r <Q-bar_r, K_t / ||K_t||> (Alg. 1, S and S-hat steps);
    the ablation variants as in key_scores."""
    assert similarity in ("cosine", "dot") and reduce in ("max", "mean")
    qbar = np.asarray(qbar, dtype=np.float64)
    Kn = np.asarray(K, dtype=np.float64)
    if similarity == "cosine":
        Kn = unit(Kn)
    n_kv, T = Kn.shape[0], Kn.shape[1]
    out = np.empty((n_kv, T), dtype=np.float64)
    for kv in range(n_kv):
        if T == 0:
            out[kv] = np.empty((0,))
        else:
            S = qbar[kv] @ Kn[kv].T
            out[kv] = S.max(axis=0) if reduce == "max" else S.mean(axis=0)
    return out


def topk_keys(scores: np.ndarray, budget: int) -> np.ndarray:
    """I [n_kv, B'] with B' = min(budget, T): the highest-scoring keys per KV head.

    Alg. 1, topk step.  Ties go to the lower position; indices are reported in
    ascending position.
    """
    scores = np.asarray(scores, dtype=np.float64)
    n_kv, T = scores.shape
    Bp = max(0, min(int(budget), T))
    out = np.empty((n_kv, Bp), dtype=np.int64)
    for kv in range(n_kv):
        order = np.argsort(-scores[kv], kind="stable")   # descending score, ties -> lower index
        out[kv] = np.sort(order[:Bp])
    return out


# ---------------------------------------------------------------------------
# Eq. 1-3 / Alg. 2: attention of the chunk over [selected past | chunk]
# ---------------------------------------------------------------------------
def _attend_head(q: np.ndarray, k_past: np.ndarray, v_past: np.ndarray,
                 k_chunk: np.ndarray, v_chunk: np.ndarray, rows=None):
    """Softmax(q [k_past | k_chunk]^T / sqrt(d) + M) [v_past | v_chunk] for one head.

    M lets every chunk query see all past keys and chunk keys at positions <= its own.
    `rows` (optional) restricts the computation to those chunk positions (same arithmetic per row).
    Returns (O [R, d], lse [R]) with lse the natural-log normaliser of each row.
    """
    C, d = q.shape
    pos = np.arange(C) if rows is None else np.asarray(rows, dtype=np.int64)
    P = k_past.shape[0]
    k_all = np.concatenate([k_past, k_chunk], axis=0)
    v_all = np.concatenate([v_past, v_chunk], axis=0)
    logits = (q[pos] @ k_all.T) / np.sqrt(d)                  # [R, P + C]
    i = pos[:, None]
    c = np.arange(C)[None, :]
    mask = np.zeros((pos.shape[0], P + C), dtype=bool)
    mask[:, P:] = c > i                                       # future chunk tokens
    logits = np.where(mask, -np.inf, logits)
    m = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - m)
    z = e.sum(axis=1, keepdims=True)
    return (e / z) @ v_all, (m + np.log(z))[:, 0]


def sparse_attn(Q, K, V, k_idx, Kc, Vc, return_lse: bool = False, rows=None, heads=None):
    """Chunk attention over gather(K, I), gather(V, I) and the chunk's own KV (Eq. 3, Alg. 2).

    k_idx: sequence of n_kv index arrays into the past cache (one per KV head).
    rows / heads (optional): compute only these chunk positions / q-heads (for sampled checks at
    sizes where the full result is too slow); outputs then have shape [len(heads), len(rows), d].
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    Kc = np.asarray(Kc, dtype=np.float64)
    Vc = np.asarray(Vc, dtype=np.float64)
    n_q, C, d = Q.shape
    n_kv = K.shape[0]
    g = n_q // n_kv
    hs = list(range(n_q)) if heads is None else [int(h) for h in heads]
    R = C if rows is None else len(rows)
    O = np.empty((len(hs), R, d), dtype=np.float64)
    L = np.empty((len(hs), R), dtype=np.float64)
    for n, h in enumerate(hs):
        kv = h // g
        idx = np.asarray(k_idx[kv], dtype=np.int64)
        O[n], L[n] = _attend_head(Q[h], K[kv][idx], V[kv][idx], Kc[kv], Vc[kv], rows)
    return (O, L) if return_lse else O


def dense_attn(Q, K, V, Kc, Vc, return_lse: bool = False, rows=None, heads=None):
    """Dense chunked-prefill attention of the chunk over the whole past cache (Eq. 2)."""
    K = np.asarray(K)
    T = K.shape[1]
    full = [np.arange(T, dtype=np.int64)] * K.shape[0]
    return sparse_attn(Q, K, V, full, Kc, Vc, return_lse, rows, heads)


def quoka_select(Q, K, n_retain: int, budget: int, similarity: str = "cosine", reduce: str = "max",
                 query_rule: str = "cosine"):
    """Alg. 1 up to the index set: returns (q_idx, scores, k_idx).  The ablation scorers change only the key
    scores; query_rule="uniform" changes only which queries are retained."""
    n_kv = np.asarray(K).shape[0]
    q_idx = select_queries(Q, n_retain, query_rule)
    scores = key_scores(Q, q_idx, K, n_kv, similarity, reduce)
    k_idx = topk_keys(scores, budget)
    return q_idx, scores, k_idx


def quoka_chunk_attn(Q, K, V, Kc, Vc, n_retain: int, budget: int):
    """One iteration of Alg. 2's loop body: select with Alg. 1, then attend.  Returns (O, k_idx)."""
    _, _, k_idx = quoka_select(Q, K, n_retain, budget)
    return sparse_attn(Q, K, V, k_idx, Kc, Vc), k_idx


def chunked_prefill(Qs, Ks, Vs, chunk: int, n_retain: int = 0, budget=None):
    """Alg. 2 over a whole sequence.  Qs [n_q, L, d], Ks/Vs [n_kv, L, d].

    budget=None runs dense chunked prefill (Eq. 2); otherwise QuoKA with that B_SA.
    The cache grows by one chunk per iteration (the update step of Alg. 2).
    """
    Qs = np.asarray(Qs, dtype=np.float64)
    Ks = np.asarray(Ks, dtype=np.float64)
    Vs = np.asarray(Vs, dtype=np.float64)
    L = Qs.shape[1]
    outs = []
    for s in range(0, L, chunk):
        e = min(s + chunk, L)
        Qi, Ki, Vi = Qs[:, s:e], Ks[:, s:e], Vs[:, s:e]
        Kp, Vp = Ks[:, :s], Vs[:, :s]
        if budget is None:
            outs.append(dense_attn(Qi, Kp, Vp, Ki, Vi))
        else:
            outs.append(quoka_chunk_attn(Qi, Kp, Vp, Ki, Vi, n_retain, budget)[0])
    return np.concatenate(outs, axis=1)
