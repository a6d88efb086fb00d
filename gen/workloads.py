"""Deterministic workload generator (numpy PCG64), CPU only.

Every tensor is returned as float32 holding values that are exactly
representable in the workload's storage dtype (fp32, or bf16 after
round-to-nearest-even), so the CPU oracle and the GPU see identical numbers.

Layouts (row-major, head_dim contiguous):
  Q        [b, n_q,  C,     d]   chunk queries
  K, V     [b, n_kv, T_max, d]   past KV cache (rows >= kv_lens[b] are padding)
  Kc, Vc   [b, n_kv, C,     d]   the chunk's own keys / values
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

CONFIG_NAMES = ("c1", "c2", "c3", "c4", "c5")


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-exact."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


@dataclass
class Workload:
    name: str
    dtype: str              # "f32" or "bf16"
    batch: int
    n_q: int
    n_kv: int
    d: int
    chunk: int              # C = B_CP
    t_max: int              # extent of the cache's token axis
    kv_lens: List[int]      # T_b per sequence
    n_retain: int           # N_Q
    budgets: List[int]      # B_SA per sequence
    seed: int
    Q: np.ndarray = field(repr=False, default=None)
    K: np.ndarray = field(repr=False, default=None)
    V: np.ndarray = field(repr=False, default=None)
    Kc: np.ndarray = field(repr=False, default=None)
    Vc: np.ndarray = field(repr=False, default=None)
    notes: dict = field(default_factory=dict)

    @property
    def group(self) -> int:
        return self.n_q // self.n_kv


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _normal(rng, shape) -> np.ndarray:
    return rng.standard_normal(size=shape, dtype=np.float32)


def _unit(rng, shape) -> np.ndarray:
    v = rng.standard_normal(size=shape).astype(np.float64)
    v /= np.linalg.norm(v, axis=-1, keepdims=True)
    return v.astype(np.float32)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    return bf16_round(x) if dtype == "bf16" else x


def _rope(x: np.ndarray, positions: np.ndarray, base: float = 5.0e5) -> np.ndarray:
    """Rotary position embedding, rotate-half pairing, applied in float64.

    x: [..., n_tok, d]; positions: [n_tok].  The base is a generator choice
    (the selection method does not depend on it).
    """
    d = x.shape[-1]
    half = d // 2
    inv_freq = base ** (-np.arange(half, dtype=np.float64) / half)
    ang = positions.astype(np.float64)[:, None] * inv_freq[None, :]
    cos, sin = np.cos(ang), np.sin(ang)
    x = x.astype(np.float64)
    x1, x2 = x[..., :half], x[..., half:]
    out = np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)
    return out.astype(np.float32)


def _offset_queries(rng, b, n_q, C, d, offset_norm):
    """N(0,1) queries plus a per-head mean direction of the given norm."""
    Q = _normal(rng, (b, n_q, C, d))
    u = _unit(rng, (b, n_q, 1, d))
    return Q + np.float32(offset_norm) * u, u


def make_custom(*, dtype="bf16", batch=1, n_q=4, n_kv=2, d=64, chunk=32, kv_lens=(100,),
                n_retain=8, budgets=(16,), seed=0, offset_norm=1.5, t_max: Optional[int] = None,
                name="custom") -> Workload:
    """Small generic workload: N(0,1) tensors, per-head query offset, no planted structure."""
    kv_lens = [int(t) for t in kv_lens]
    budgets = [int(x) for x in budgets]
    assert len(kv_lens) == batch and len(budgets) == batch
    t_max = int(t_max if t_max is not None else max(max(kv_lens), 1))
    rng = _rng(seed)
    Q, _ = _offset_queries(rng, batch, n_q, chunk, d, offset_norm)
    K = _normal(rng, (batch, n_kv, t_max, d))
    V = _normal(rng, (batch, n_kv, t_max, d))
    Kc = _normal(rng, (batch, n_kv, chunk, d))
    Vc = _normal(rng, (batch, n_kv, chunk, d))
    return Workload(name, dtype, batch, n_q, n_kv, d, chunk, t_max, kv_lens, n_retain, budgets, seed,
                    _store(Q, dtype), _store(K, dtype), _store(V, dtype), _store(Kc, dtype), _store(Vc, dtype))


def _c1() -> Workload:
    # Tiny fp32 case with planted structure.  Built by construction (no ranking here):
    # 16 queries of head 0 are drawn away from the shared mean direction, and 8 cache
    # keys are set parallel to 8 of them with norm sqrt(d).
    b, n_q, n_kv, d, T, C, n_ret, B, seed = 1, 2, 1, 64, 1024, 128, 16, 128, 0
    rng = _rng(seed)
    Q = _normal(rng, (b, n_q, C, d))
    K = _normal(rng, (b, n_kv, T, d))
    V = _normal(rng, (b, n_kv, T, d))
    Kc = _normal(rng, (b, n_kv, C, d))
    Vc = _normal(rng, (b, n_kv, C, d))
    u = _unit(rng, (d,))
    Q = Q + np.float32(2.0) * u
    out_pos = np.sort(rng.choice(C, size=n_ret, replace=False))
    eps = _normal(rng, (n_ret, d))
    # outliers: remove the component along u, then push four units against it
    Q[0, 0, out_pos] = eps - (eps @ u)[:, None] * u - np.float32(4.0) * u
    heavy_q = np.sort(rng.choice(out_pos, size=8, replace=False))
    heavy_pos = np.sort(rng.choice(T, size=8, replace=False))
    qh = Q[0, 0, heavy_q].astype(np.float64)
    K[0, 0, heavy_pos] = (np.sqrt(d) * qh / np.linalg.norm(qh, axis=-1, keepdims=True)).astype(np.float32)
    w = Workload("c1", "f32", b, n_q, n_kv, d, C, T, [T], n_ret, [B], seed, Q, K, V, Kc, Vc)
    w.notes = {"outlier_queries_head0": out_pos.tolist(), "heavy_key_pos": heavy_pos.tolist(),
               "heavy_query_pos": heavy_q.tolist()}
    return w


def _c2() -> Workload:
    b, n_q, n_kv, d, T, C, n_ret, seed = 1, 32, 8, 128, 8192, 1024, 64, 1
    B = int(0.12 * T)
    rng = _rng(seed)
    Q, _ = _offset_queries(rng, b, n_q, C, d, 1.5)
    K = _normal(rng, (b, n_kv, T, d))
    V = _normal(rng, (b, n_kv, T, d))
    Kc = _normal(rng, (b, n_kv, C, d))
    Vc = _normal(rng, (b, n_kv, C, d))
    past, cur = np.arange(T), np.arange(T, T + C)
    Q, K, Kc = _rope(Q, cur), _rope(K, past), _rope(Kc, cur)
    dt = "bf16"
    return Workload("c2", dt, b, n_q, n_kv, d, C, T, [T], n_ret, [B], seed,
                    _store(Q, dt), _store(K, dt), _store(V, dt), _store(Kc, dt), _store(Vc, dt))


def _c3() -> Workload:
    b, n_q, n_kv, d, T, C, n_ret, seed = 1, 32, 8, 128, 32768, 2048, 128, 2
    B = int(0.12 * T)
    rng = _rng(seed)
    Q, _ = _offset_queries(rng, b, n_q, C, d, 1.5)
    centres = _normal(rng, (b, n_kv, 16, d))
    z = rng.integers(0, 16, size=(b, n_kv, T))
    zc = rng.integers(0, 16, size=(b, n_kv, C))
    K = np.take_along_axis(centres, z[..., None], axis=2) + np.float32(0.5) * _normal(rng, (b, n_kv, T, d))
    Kc = np.take_along_axis(centres, zc[..., None], axis=2) + np.float32(0.5) * _normal(rng, (b, n_kv, C, d))
    V = _normal(rng, (b, n_kv, T, d))
    Vc = _normal(rng, (b, n_kv, C, d))
    dt = "bf16"
    return Workload("c3", dt, b, n_q, n_kv, d, C, T, [T], n_ret, [B], seed,
                    _store(Q, dt), _store(K, dt), _store(V, dt), _store(Kc, dt), _store(Vc, dt))


def _c4() -> Workload:
    b, n_q, n_kv, d, T, C, n_ret, B, seed = 1, 32, 8, 128, 131072, 4096, 128, 8192, 3
    rng = _rng(seed)
    Q, u = _offset_queries(rng, b, n_q, C, d, 1.5)
    orth = rng.random((b, n_q, C)) < 0.10
    eps = _normal(rng, (b, n_q, C, d))
    eps = eps - np.sum(eps * u, axis=-1, keepdims=True) * u
    Q = np.where(orth[..., None], eps, Q)
    K = _normal(rng, (b, n_kv, T, d))
    V = _normal(rng, (b, n_kv, T, d))
    Kc = _normal(rng, (b, n_kv, C, d))
    Vc = _normal(rng, (b, n_kv, C, d))
    dt = "bf16"
    return Workload("c4", dt, b, n_q, n_kv, d, C, T, [T], n_ret, [B], seed,
                    _store(Q, dt), _store(K, dt), _store(V, dt), _store(Kc, dt), _store(Vc, dt))


def _c5(n_retain: int = 64, budget_frac: float = 0.12) -> Workload:
    b, n_q, n_kv, d, C, seed = 8, 32, 8, 128, 512, 4
    rng = _rng(seed)
    kv_lens = [int(t) for t in rng.integers(4096, 65536 + 1, size=b)]
    t_max = max(kv_lens)
    Q, _ = _offset_queries(rng, b, n_q, C, d, 1.5)
    K = _normal(rng, (b, n_kv, t_max, d))
    V = _normal(rng, (b, n_kv, t_max, d))
    Kc = _normal(rng, (b, n_kv, C, d))
    Vc = _normal(rng, (b, n_kv, C, d))
    budgets = [int(budget_frac * t) for t in kv_lens]
    dt = "bf16"
    return Workload("c5", dt, b, n_q, n_kv, d, C, t_max, kv_lens, n_retain, budgets, seed,
                    _store(Q, dt), _store(K, dt), _store(V, dt), _store(Kc, dt), _store(Vc, dt))


def make_workload(name: str, **kw) -> Workload:
    """Build one of the five named workloads ("c1".."c5").

    c5 accepts n_retain in {32, 64, 128} and budget_frac in {0.04, 0.12, 0.25, 1.0}.
    """
    if name == "c1":
        return _c1()
    if name == "c2":
        return _c2()
    if name == "c3":
        return _c3()
    if name == "c4":
        return _c4()
    if name == "c5":
        return _c5(**kw)
    raise ValueError(f"unknown workload {name!r}")
