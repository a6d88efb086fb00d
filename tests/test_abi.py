"""Host-side checks of the C ABI: the library loads, exports every declared symbol, and rejects bad
arguments before launching anything (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pk():
    import paper_2602_08722_amd as pk
    pk.load_library()
    return pk


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "quoka.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(quoka_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(pk):
    lib = pk.load_library()
    names = _declared_symbols()
    assert set(names) >= {"quoka_select_queries", "quoka_score_keys", "quoka_topk_keys", "quoka_sparse_attn",
                          "quoka_dense_attn", "quoka_chunk_attn", "quoka_workspace_bytes"}
    for n in names:
        assert hasattr(lib, n), n
    from paper_2602_08722_amd.binding import EXPORTS
    assert sorted(EXPORTS) == names


def _shape(pk, **kw):
    s = pk.QuokaShape()
    vals = dict(batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, chunk_len=64, max_kv_len=1000, n_retain=16,
                max_budget=100, dtype=pk.QUOKA_BF16, score_flags=0)
    vals.update(kw)
    for k, v in vals.items():
        setattr(s, k, v)
    d = vals["head_dim"]
    for name, tok in (("q_stride", vals["chunk_len"]), ("kv_stride", max(vals["max_kv_len"], 1)),
                      ("ck_stride", vals["chunk_len"]), ("o_stride", vals["chunk_len"])):
        heads = vals["n_q_heads"] if name in ("q_stride", "o_stride") else vals["n_kv_heads"]
        setattr(s, name, (ctypes.c_int64 * 3)(heads * tok * d, tok * d, d))
    return s


def _ws_status(pk, s):
    n = ctypes.c_size_t(0)
    return pk.load_library().quoka_workspace_bytes(ctypes.byref(s), ctypes.byref(n)), n.value


def test_struct_layout_matches_header(pk):
    # 10 int32 then 4 x 3 int64
    assert ctypes.sizeof(pk.QuokaShape) == 10 * 4 + 12 * 8
    assert pk.QuokaShape.q_stride.offset == 40


def test_workspace_query_and_status_strings(pk):
    st, n = _ws_status(pk, _shape(pk))
    assert st == 0 and n > 0 and n % 256 == 0
    st2, n2 = _ws_status(pk, _shape(pk, max_kv_len=100000, max_budget=5000))
    assert st2 == 0 and n2 > n          # the multi-block top-k path needs histogram space
    lib = pk.load_library()
    assert lib.quoka_status_string(0) == b"ok"
    assert all(lib.quoka_status_string(i) for i in range(6))
    assert pk.quoka_version() >= 100


@pytest.mark.parametrize("kw,code", [
    (dict(n_q_heads=6, n_kv_heads=4), 1),          # not divisible
    (dict(batch=0), 1),
    (dict(chunk_len=0), 1),
    (dict(n_retain=0), 1),
    (dict(max_budget=2000), 1),                    # budget extent beyond the cache extent
    (dict(score_flags=32), 1),
    (dict(head_dim=96), 2),
    (dict(dtype=7), 2),
    (dict(n_retain=129), 2),
    (dict(chunk_len=8193), 2),
    (dict(n_q_heads=34, n_kv_heads=2), 2),           # more than 16 q-heads per KV head
])
def test_bad_shapes_are_rejected(pk, kw, code):
    st, _ = _ws_status(pk, _shape(pk, **kw))
    assert st == code


def test_bad_strides_and_null_pointers_are_rejected_without_a_launch(pk):
    lib = pk.load_library()
    s = _shape(pk)
    s.q_stride[2] = 100            # not a multiple of 8
    assert _ws_status(pk, s)[0] == 1
    s = _shape(pk)
    s.kv_stride[2] = 64            # rows would overlap
    assert _ws_status(pk, s)[0] == 1
    s = _shape(pk)
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: every call below must fail validation first
    ws_ok = ctypes.c_void_p(0x10000)
    big = ctypes.c_size_t(1 << 30)
    assert lib.quoka_select_queries(ctypes.byref(s), None, fake, fake, ws_ok, big, None) == 1
    assert lib.quoka_select_queries(ctypes.byref(s), fake, fake, fake, None, big, None) == 1
    assert lib.quoka_select_queries(ctypes.byref(s), fake, fake, fake, ws_ok, ctypes.c_size_t(16), None) == 3
    assert lib.quoka_select_queries(ctypes.byref(s), fake, fake, fake, ctypes.c_void_p(0x10010), big, None) == 3
    assert lib.quoka_select_queries(ctypes.byref(s), ctypes.c_void_p(0x1004), fake, fake, ws_ok, big, None) == 1
    assert lib.quoka_score_keys(ctypes.byref(s), fake, None, fake, fake, ws_ok, big, None) == 1
    assert lib.quoka_topk_keys(ctypes.byref(s), fake, fake, None, fake, fake, ws_ok, big, None) == 1
    assert lib.quoka_sparse_attn(ctypes.byref(s), fake, fake, fake, None, fake, fake, fake, fake, None, ws_ok, big,
                                 None) == 1
    assert lib.quoka_dense_attn(ctypes.byref(s), fake, fake, fake, None, fake, fake, fake, None, ws_ok, big,
                                None) == 1
    assert lib.quoka_chunk_attn(ctypes.byref(s), None, fake, fake, fake, fake, fake, fake, fake, fake, fake, fake,
                                fake, fake, None, ws_ok, big, None) == 1
    assert lib.quoka_prefill_attn(ctypes.byref(s), 1, fake, None, fake, fake, fake, fake, fake, fake, fake, fake, fake,
                                  ws_ok, big, None) == 1
    assert lib.quoka_prefill_attn(ctypes.byref(s), 1, fake, fake, fake, fake, None, fake, fake, fake, fake, fake, fake,
                                  ws_ok, big, None) == 1   # sparse prefill needs budgets
    assert lib.quoka_workspace_bytes(None, ctypes.byref(ctypes.c_size_t(0))) == 1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2602_08722_amd.binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "library_path", lambda: str(tmp_path / "libquoka.so"))
    with pytest.raises(FileNotFoundError):
        B.load_library()


def test_bench_refuses_more_than_one_gpu():
    """This build is single-GPU: `bench.py --gpus N` with N > 1 must exit with a message, before touching a GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "single-GPU" in r.stderr


def test_product_path_never_touches_the_oracle():
    """The package (binding, build script, kernels) must not import, read or link anything under oracle/."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2602_08722_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f), encoding="utf-8").read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"


def test_flag_and_enum_values_match_the_header(pk):
    """The Python constants are typed in by hand: check them against the declarations in include/quoka.h."""
    text = open(os.path.join(ROOT, "include", "quoka.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    vals = {m.group(1): int(m.group(2)) for m in re.finditer(r"\b(QUOKA_[A-Z0-9_]+)\s*=\s*(\d+)", text)}
    for name in ("QUOKA_F32", "QUOKA_BF16", "QUOKA_SCORE_DOT", "QUOKA_SCORE_MEAN", "QUOKA_SELECT_UNIFORM",
                 "QUOKA_SCORE_QBAR_BF16", "QUOKA_ATTN_SCALE_F32"):
        assert name in vals, name
        assert getattr(pk, name) == vals[name], name
    flags = [v for k, v in vals.items() if k.startswith(("QUOKA_SCORE_", "QUOKA_SELECT_", "QUOKA_ATTN_"))]
    assert sorted(flags) == [1, 2, 4, 8, 16]       # distinct single bits
    # every flag bit is accepted, the next bit is not
    assert _ws_status(pk, _shape(pk, score_flags=31))[0] == 0
    assert _ws_status(pk, _shape(pk, score_flags=32))[0] == 1
