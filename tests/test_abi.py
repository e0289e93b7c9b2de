"""Host-side checks of the C ABI that need no GPU: exports, argument validation, error strings."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2503_00784_amd import binding as B
from paper_2503_00784_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2503_00784_amd import build
        build.build(verbose=False)
    return B.load()


def test_every_declared_entry_point_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "duo_verify.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(duo_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for dtype in ("bf16", "fp16"):  # the two builds of the same sources export the same entry points
        one = B.load(dtype)
        for name in declared:
            assert getattr(one, name) is not None


def test_status_strings(lib):
    assert B.status_string(0) == "ok"
    seen = {B.status_string(c) for c in range(-9, 1)}
    assert len(seen) == 10 and "unknown status" not in seen
    assert B.status_string(-99) == "unknown status"


def test_workspace_bytes_validation(lib):
    cfg = B.make_config(inputs.TINY, 256)
    n = B.workspace_bytes(cfg, 8)
    assert n > 16 * 768 * 4 + 16 * 32000 * 4
    assert B.workspace_bytes(cfg, 80) > n
    out = C.c_size_t()
    assert lib.duo_workspace_bytes(None, 8, C.byref(out)) == -1
    assert lib.duo_workspace_bytes(C.byref(cfg), 8, None) == -1
    assert lib.duo_workspace_bytes(C.byref(cfg), 0, C.byref(out)) == -2
    assert lib.duo_workspace_bytes(C.byref(cfg), 81, C.byref(out)) == 0      # prompt chunks take up to 1024 rows
    assert lib.duo_workspace_bytes(C.byref(cfg), 1024, C.byref(out)) == 0 and out.value > n
    assert lib.duo_workspace_bytes(C.byref(cfg), 1025, C.byref(out)) == -2
    for field, bad in [("head_dim", 96), ("d_model", 770), ("max_seq", 250), ("n_kv_heads", 5), ("d_ff", 100)]:
        c2 = B.make_config(inputs.TINY, 256)
        setattr(c2, field, bad)
        assert lib.duo_workspace_bytes(C.byref(c2), 8, C.byref(out)) == -2, field


def _fake_weights(n_layers, addr=0x1000):
    tabs = {}
    w = B.Weights()
    w.embed = w.lm_head = w.g_final = addr
    for key in B._LAYER_KEYS:
        tab = (C.c_void_p * n_layers)(*([addr] * n_layers))
        tabs[key] = tab
        setattr(w, key, C.cast(tab, C.POINTER(C.c_void_p)))
    return w, tabs


def test_verify_rejects_bad_arguments_before_touching_the_gpu(lib):
    """Every call below must fail validation on the host; none may enqueue work (there is no GPU here)."""
    cfg = B.make_config(inputs.TINY, 256)
    w, keep = _fake_weights(cfg.n_layers)
    cache = B.KVCache(0x1000, 0x1000, 0x1000, 0x1000)
    res = B.Result(0x1000, 0x1000, 0x1000, 0x1000, None)
    ws_bytes = B.workspace_bytes(cfg, 80)

    def run(call, cfg=cfg, w=w, cache=cache, res=res, toks=0x1000, q=0x1000, u=0x1000, ws=0x1000, nbytes=ws_bytes):
        return lib.duo_verify(C.byref(cfg), C.byref(w) if w else None, C.byref(cache) if cache else None, toks, q, u,
                              C.byref(call) if call else None, C.byref(res) if res else None, ws, nbytes, None)

    good = B.Call(1, 8, 1.0, 0, -1, 128)
    assert run(None) == -1
    assert run(good, w=None) == -1
    assert run(good, cache=None) == -1
    assert run(good, res=None) == -1
    assert run(good, toks=None) == -1 and run(good, q=None) == -1 and run(good, u=None) == -1 and run(good, ws=None) == -1
    assert run(good, cache=B.KVCache(0x1000, 0x1000, 0x1000, None)) == -1      # no root logits, no root token
    assert run(B.Call(0, 8, 1.0, 0, -1, 128)) == -2
    assert run(B.Call(1, 0, 1.0, 0, -1, 128)) == -2
    assert run(B.Call(10, 8, 1.0, 0, 5, 128)) == -2                            # 81 rows with the root
    assert run(B.Call(11, 8, 1.0, 0, -1, 128)) == -2
    assert run(B.Call(1, 8, -0.5, 0, -1, 128)) == -8                           # 0 is the greedy limit, below it nothing
    assert run(B.Call(1, 8, float("nan"), 0, -1, 128)) == -8
    assert run(B.Call(1, 8, 1.0, 2, -1, 128)) == -8
    assert run(B.Call(1, 8, 1.0, 0, 32000, 128)) == -6
    assert run(B.Call(1, 8, 1.0, 0, -1, 249)) == -3                            # 249 + 8 > 256
    assert run(B.Call(1, 8, 1.0, 0, -1, 248), ws=0x1008) == -4
    assert run(B.Call(1, 8, 1.0, 0, -1, 248), q=0x1004) == -4
    assert run(B.Call(1, 8, 1.0, 0, -1, 248), nbytes=ws_bytes // 100) == -5
    w2, keep2 = _fake_weights(cfg.n_layers)
    keep2["wo"][1] = None
    assert run(good, w=w2) == -1
    keep2["wo"][1] = 0x1002
    assert run(good, w=w2) == -4


def test_other_entry_points_validate(lib):
    cfg = B.make_config(inputs.TINY, 256)
    w, keep = _fake_weights(cfg.n_layers)
    cache = B.KVCache(0x1000, 0x1000, 0x1000, 0x1000)
    nbytes = B.workspace_bytes(cfg, 80)
    pf = lambda m, P, toks=0x1000: lib.duo_prefill_chunk(C.byref(cfg), C.byref(w), C.byref(cache), toks, m, P, 0x1000,
                                                         0x1000, nbytes, None)
    assert pf(0, 0) == -2 and pf(1025, 0) == -2 and pf(8, 250) == -3 and pf(8, -1) == -8 and pf(8, 0, None) == -1
    out = C.c_size_t()
    assert lib.duo_sample_workspace_bytes(32000, 1, 8, C.byref(out)) == 0 and out.value >= 32000 * 8
    assert lib.duo_sample_workspace_bytes(1, 1, 8, C.byref(out)) == -2
    assert lib.duo_sample_workspace_bytes(32000, 9, 9, C.byref(out)) == -2
    call = B.Call(1, 8, 1.0, 0, -1, 0)
    res = B.Result(0x1000, 0x1000, 0x1000, 0x1000, None)
    ss = lambda **kw: lib.duo_spec_sample(kw.get("lg", 0x1000), kw.get("root", 0x1000), kw.get("V", 32000), 0x1000, 0x1000,
                                          0x1000, C.byref(call), C.byref(res), 0x1000, kw.get("nb", out.value), None)
    assert ss(lg=None) == -1 and ss(root=None) == -1 and ss(V=1) == -2 and ss(nb=16) == -5
    # the entry point without a workspace: same checks, plus the limits of its static scratch (all before any GPU call)
    na = lambda **kw: lib.duo_spec_sample_noalloc(kw.get("lg", 0x1000), kw.get("root", 0x1000), kw.get("V", 32000), 0x1000,
                                                  kw.get("q", 0x1000), 0x1000, C.byref(kw.get("call", call)), C.byref(res), None)
    assert na(lg=None) == -1 and na(root=None) == -1 and na(q=None) == -1 and na(V=1) == -2
    assert na(V=B.NOALLOC_MAX_VOCAB + 1) == -9
    assert na(call=B.Call(1, 8, 1.0, 0, -1, 0, 0.9)) == -9            # the nucleus search needs rows the scratch does not hold
    assert na(call=B.Call(1, 0, 1.0, 0, -1, 0)) == -2 and na(call=B.Call(1, 8, -1.0, 0, -1, 0)) == -8
    # the deferred form takes an empty suffix (k = 0) but no negative one; n must be 1
    ds = lambda c, **kw: lib.duo_deferred_sample(kw.get("lg", 0x1000), 0x1000, 32000, kw.get("toks", 0x1000), 0x1000, kw.get("u", 0x1000),
                                                 None, None, None, 0, C.byref(c), C.byref(res), 0x1000, out.value, None)
    assert ds(B.Call(1, -1, 1.0, 1, -1, 0)) == -2 and ds(B.Call(2, 4, 1.0, 1, -1, 0)) == -2
    assert ds(B.Call(1, 4, 1.0, 1, -1, 0), toks=None) == -1 and ds(B.Call(1, 0, 1.0, 1, -1, 0), u=None) == -1
    assert lib.duo_sample_workspace_bytes(32000, 1, 0, C.byref(out)) == 0
    g = lambda **kw: lib.duo_skinny_gemm(kw.get("x", 0x1000), 0x1000, 0x1000, kw.get("rows", 8), 64, kw.get("K", 64), None)
    assert g(x=None) == -1 and g(rows=0) == -2 and g(rows=81) == -2 and g(K=48) == -2 and g(x=0x1002) == -4
    assert lib.duo_packed_elems(4099, 512) == 4128 * 512 and lib.duo_packed_elems(32, 64) == 32 * 64
    assert lib.duo_packed_elems(0, 64) == 0
    pm = lambda **kw: lib.duo_pack_matrix(kw.get("src", 0x1000), kw.get("N", 64), kw.get("K", 64), kw.get("dst", 0x1000), None)
    assert pm(src=None) == -1 and pm(dst=None) == -1 and pm(N=0) == -2 and pm(K=40) == -2 and pm(src=0x1004) == -4
    assert lib.duo_pack_qkv(C.byref(cfg), None, 0x1000, 0x1000, 0x1000, None) == -1
    assert lib.duo_pack_qkv(C.byref(cfg), 0x1000, 0x1000, 0x1008, 0x1000, None) == -4
    assert lib.duo_pack_gate_up(C.byref(cfg), 0x1000, None, 0x1000, None) == -1
    bg = lambda **kw: lib.duo_block_gemm(kw.get("x", 0x1000), 0x1000, 0x1000, kw.get("rows", 256), 64, kw.get("K", 64), None)
    assert bg(x=None) == -1 and bg(rows=0) == -2 and bg(rows=1025) == -2 and bg(K=48) == -2 and bg(x=0x1002) == -4
    sp = lambda **kw: lib.duo_stream_read_probe(kw.get("src", 0x1000), kw.get("nbytes", 1 << 20), kw.get("sink", 0x1000), kw.get("n", 64), kw.get("nt", 0), None)
    assert sp(src=None) == -1 and sp(sink=None, nt=1) == -1 and sp(nbytes=8) == -2 and sp(n=0) == -2 and sp(src=0x1004) == -4
    assert lib.duo_pack_activations(0x1000, 2049, 64, 0x1000, None) == -2 and lib.duo_pack_activations(None, 8, 64, 0x1000, None) == -1


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_libs", {})
    monkeypatch.setattr(B, "LIB_PATHS", {"bf16": str(tmp_path / "nope.so"), "fp16": str(tmp_path / "nope16.so")})
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.load()
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.load("fp16")


def test_input_generators_are_seeded_and_shaped():
    w1 = inputs.make_weights(inputs.MID, seed=3, threads=2)
    w2 = inputs.make_weights(inputs.MID, seed=3, threads=4)
    assert w1["wq"][1].shape == (512, 512) and w1["w_down"][0].shape == (512, 1408) and w1["lm_head"].shape == (4099, 512)
    np.testing.assert_array_equal(w1["w_up"][2], w2["w_up"][2])
    assert not np.array_equal(w1["w_up"][2], w1["w_up"][1])
    q, t, u = inputs.make_draft(1000, 3, 4, seed=1, easy_rows=inputs.easy_rows_for(3, 4))
    assert q.shape == (3, 4, 1000) and t.shape == (3, 4) and u.shape == (3, 5)
    np.testing.assert_allclose(q.sum(-1), 1.0, rtol=1e-5)
    assert u.min() >= 0.0 and u.max() < 1.0 and t.min() >= 0 and t.max() < 1000
    wl = inputs.WORKLOADS["C3"]
    assert abs(wl.algorithmic_bytes() / 1e9 - 15.362) < 0.005 and abs(wl.shape.weight_bytes() / 1e9 - 13.214) < 0.005
    assert abs(inputs.WORKLOADS["C1"].algorithmic_bytes() / 1e9 - 13.483) < 0.005


@pytest.mark.parametrize("D", [64, 128])
def test_kv_cache_layout_formulas_agree_with_the_binding(D):
    """The tiled KV-cache layouts: the library's host-side offset functions, the formulas printed in the header and
    the binding's reshapes address the same element; the reshapes are inverses of each other."""
    import torch
    lib = B.load()
    S = 96
    rows = torch.arange(S * D, dtype=torch.int32).reshape(1, 1, S, D)  # unique values, leading [layer][head] axes
    kt, vt = B.k_rows_to_tiles(rows), B.v_rows_to_tiles(rows)
    assert kt.shape == (1, 1, S * D) and vt.shape == (1, 1, S * D)
    g = np.random.default_rng(D)
    for slot, d in zip(g.integers(0, S, 200), g.integers(0, D, 200)):
        slot, d = int(slot), int(d)
        Bk, w = slot // 32, slot % 32
        t = (w % 8) // 4
        k_off = ((((Bk * 2 + t) * (D // 32) + d // 32) * 64 + ((d % 32) // 8) * 16 + 4 * (w // 8) + w % 4) * 8 + d % 8)
        v_off = (((Bk * (D // 16) + d // 16) * 64 + (w // 8) * 16 + d % 16) * 8 + w % 8)
        assert lib.duo_k_cache_offset(D, slot, d) == k_off
        assert lib.duo_v_cache_offset(D, slot, d) == v_off
        assert int(kt[0, 0, k_off]) == int(rows[0, 0, slot, d])
        assert int(vt[0, 0, v_off]) == int(rows[0, 0, slot, d])
    assert torch.equal(B.k_tiles_to_rows(kt, D), rows)
    assert torch.equal(B.v_tiles_to_rows(vt, D), rows)
    # every offset is hit exactly once
    assert sorted(kt.flatten().tolist()) == sorted(rows.flatten().tolist())


def test_header_is_valid_c99_and_cxx():
    """The boundary is a C ABI: the header must compile on its own as C and as C++."""
    import shutil
    import subprocess
    hdr = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "duo_verify.h")
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", hdr], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", hdr], check=True)
