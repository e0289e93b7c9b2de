"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest

from oracle import duo_oracle as O
from paper_2503_00784_amd import inputs
from tests.gpu_util import (ACCEPT_TIE, compare_end_to_end, logits_close, same_as_sampler_on, say, to_dev)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2503_00784_amd import binding
    binding.load()
    return binding


# ------------------------------------------------------------------ skinny GEMM
@pytest.mark.parametrize("rows,N,K", [(1, 64, 64), (8, 4096, 4096), (16, 1000, 512), (33, 4099, 1408), (64, 11008, 4096),
                                      (65, 4096, 11008), (80, 515, 96), (7, 17, 32)])
def test_skinny_gemm_matches_oracle_matmul(B, rows, N, K):
    import torch
    say(f"gemm rows={rows} N={N} K={K}")
    g = np.random.default_rng(rows * 1000 + N)
    x = inputs.f32_to_bf16_bits(g.normal(0, 1, (rows, K)).astype(np.float32))
    w = inputs.f32_to_bf16_bits(g.normal(0, 0.02, (N, K)).astype(np.float32))
    y = B.skinny_gemm(to_dev(x.view(np.int16)), to_dev(w.view(np.int16)))
    torch.cuda.synchronize()
    ref = O.bf16_bits_to_f64(x) @ O.bf16_bits_to_f64(w).T
    err = np.abs(y.cpu().numpy() - ref).max()
    say(f"  max abs err {err:.3e}")
    # fp32 accumulation of K products of magnitude ~0.02: error far below 1e-4 * sqrt(K)
    assert err <= 2e-6 * np.sqrt(K) * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("rows,N,K", [(81, 128, 64), (128, 4096, 4096), (256, 1000, 512), (300, 4099, 1408), (1024, 520, 2048),
                                      (130, 96, 96), (512, 11008, 4096), (255, 4096, 11008)])
def test_block_gemm_matches_oracle_matmul(B, rows, N, K):
    """The many-row projection kernel: activations as bf16 pairs (hi + lo), several row blocks, ragged rows, bands
    and K steps."""
    import torch
    say(f"block gemm rows={rows} N={N} K={K}")
    g = np.random.default_rng(rows * 1000 + N)
    a = g.normal(0, 1, (rows, K)).astype(np.float32)
    hi = inputs.f32_to_bf16_bits(a)
    lo = inputs.f32_to_bf16_bits((a.astype(np.float64) - O.bf16_bits_to_f64(hi)).astype(np.float32))
    w = inputs.f32_to_bf16_bits(g.normal(0, 0.02, (N, K)).astype(np.float32))
    y = B.block_gemm(to_dev(hi.view(np.int16)), to_dev(lo.view(np.int16)), to_dev(w.view(np.int16)))
    torch.cuda.synchronize()
    ref = (O.bf16_bits_to_f64(hi) + O.bf16_bits_to_f64(lo)) @ O.bf16_bits_to_f64(w).T
    err = np.abs(y.cpu().numpy() - ref).max()
    say(f"  max abs err {err:.3e}")
    assert err <= 2e-6 * np.sqrt(K) * max(1.0, np.abs(ref).max())


# ------------------------------------------------------------------ sampler on identical logits
def _sampling_case(V, n, k, seed, has_root, peaked):
    g = np.random.default_rng(seed)
    R = 1 if has_root else 0
    scale = 4.0 if peaked else 1.28
    logits = (g.normal(0, scale, (R + n * k, V))).astype(np.float32)
    root = (g.normal(0, scale, V)).astype(np.float32)
    q, toks, u = inputs.make_draft(V, n, k, seed=seed, easy_rows=inputs.easy_rows_for(n, k))
    if peaked:  # make drafts agree with the target often: draft tokens = argmax of the judging row
        for i in range(n):
            for j in range(k):
                if g.random() < 0.7:
                    jr = (logits[0] if has_root else root) if j == 0 else logits[R + i * k + j - 1]
                    toks[i, j] = int(np.argmax(jr))
    return logits, root, q, toks, u


@pytest.mark.parametrize("V,n,k,has_root,peaked", [(32000, 1, 8, False, False), (32000, 4, 8, False, True),
                                                    (32000, 8, 8, True, True), (4099, 3, 5, True, False),
                                                    (128256, 4, 16, False, True), (50, 2, 3, False, False),
                                                    (1031, 1, 1, False, True), (32000, 1, 16, True, True),
                                                    (8200, 3, 5, False, False), (12345, 80, 1, False, True),
                                                    (8192, 13, 6, True, True)])
@pytest.mark.parametrize("mode", [0, 1])
def test_sampler_bit_exact_on_identical_logits(B, V, n, k, has_root, peaked, mode):
    """Vocabularies below 8192 entries take the one-workgroup-per-sequence kernel, the others the kernels that cut the
    vocabulary into slices: 8192 and 8200 (two slices, a ragged last chunk), 12345 with 80 sequences (one slice each),
    32000 (seven slices), 128256 (thirty-one)."""
    total = ties = 0
    for seed in range(3):
        say(f"sampler V={V} n={n} k={k} root={has_root} peaked={peaked} mode={mode} seed={seed}")
        logits, root, q, toks, u = _sampling_case(V, n, k, seed, has_root, peaked)
        ref = O.speculative_verify(logits, root, toks, q, u, prefix_len=100, temperature=0.9 if seed == 2 else 1.0,
                                   select_mode=mode, has_root=has_root)
        got = B.spec_sample(to_dev(logits), to_dev(root), to_dev(toks), to_dev(q), to_dev(u),
                            temperature=0.9 if seed == 2 else 1.0, select_mode=mode, has_root=has_root, prefix_len=100)
        assert got["status"] == 0
        total += 1
        if ref.commit_margin <= 1e-9 or (mode == 0 and min(ref.accept_margins.min(), ref.draw_margins.min()) <= 1e-9):
            ties += 1
            continue
        np.testing.assert_array_equal(got["accept_len"], ref.accept_len)
        np.testing.assert_array_equal(got["next_token"], ref.next_token)
        assert (got["selected"], got["commit_len"], got["commit_token"], got["new_prefix_len"]) == \
               (ref.selected, ref.commit_len, ref.commit_token, ref.new_prefix_len)
    assert ties < total


@pytest.mark.parametrize("V,n,k,has_root", [(32000, 1, 8, False), (32000, 4, 8, True), (4099, 3, 5, False),
                                            (128256, 2, 16, False), (50, 2, 3, True), (8200, 3, 5, True)])
@pytest.mark.parametrize("mode", [0, 1])
def test_sampler_greedy_limit_bit_exact(B, V, n, k, has_root, mode):
    """Temperature 0: one-hot target distributions (arg max, lowest id among equal logits) on both sides."""
    for seed in range(3):
        say(f"greedy sampler V={V} n={n} k={k} root={has_root} mode={mode} seed={seed}")
        logits, root, q, toks, u = _sampling_case(V, n, k, seed, has_root, True)
        if seed == 2:  # equal largest logits in every row, some of them across the sampler's vocabulary slices
            for r in range(logits.shape[0]):
                a = int(np.argmax(logits[r]))
                logits[r, (a + V // 2) % V] = logits[r, a]
                logits[r, (a + 1) % V] = logits[r, a]
            root[(int(np.argmax(root)) + V // 3) % V] = root.max()
        ref = O.speculative_verify(logits, root, toks, q, u, prefix_len=100, temperature=0.0, select_mode=mode,
                                   has_root=has_root)
        got = B.spec_sample(to_dev(logits), to_dev(root), to_dev(toks), to_dev(q), to_dev(u), temperature=0.0,
                            select_mode=mode, has_root=has_root, prefix_len=100)
        assert got["status"] == 0
        np.testing.assert_array_equal(got["accept_len"], ref.accept_len)
        np.testing.assert_array_equal(got["next_token"], ref.next_token)
        assert (got["selected"], got["commit_len"], got["commit_token"], got["new_prefix_len"]) == \
               (ref.selected, ref.commit_len, ref.commit_token, ref.new_prefix_len)


def _nucleus_margin(logits, root, has_root, n, k, T, top_p):
    """Smallest distance of a running mass from the nucleus cut over all judging rows (see oracle.nucleus)."""
    rows = [logits[0] if has_root else root] + [logits[(1 if has_root else 0) + r] for r in range(n * k)]
    return min(O.nucleus(O.target_probs(r, T), top_p)[1] for r in rows)


@pytest.mark.parametrize("V,n,k,has_root,peaked", [(32000, 1, 8, False, False), (32000, 4, 8, True, True), (4099, 3, 5, False, True),
                                                    (128256, 2, 16, False, True), (50, 2, 3, True, False)])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("top_p", [0.9, 0.35])
def test_sampler_top_p_bit_exact_on_identical_logits(B, V, n, k, has_root, peaked, mode, top_p):
    """Nucleus restriction of the target distributions on both sides; decisions whose margin (accept test, draw,
    or the running mass at the nucleus cut) is within rounding of a tie are not compared."""
    total = ties = 0
    for seed in range(3):
        T = 0.8 if seed == 1 else 1.0
        say(f"top-p sampler V={V} n={n} k={k} root={has_root} peaked={peaked} mode={mode} top_p={top_p} seed={seed}")
        logits, root, q, toks, u = _sampling_case(V, n, k, seed, has_root, peaked)
        if seed == 2:  # several equal logits around the cut of the first rows: the ascending-id rule decides
            for r in range(min(3, logits.shape[0])):
                order = np.argsort(-logits[r])
                full = O.target_probs(logits[r], T)
                m = int(np.searchsorted(np.cumsum(full[order]), top_p))
                grp = order[max(0, m - 2):m + 3]
                logits[r, grp] = logits[r, order[m]]
        ref = O.speculative_verify(logits, root, toks, q, u, prefix_len=100, temperature=T, select_mode=mode,
                                   has_root=has_root, top_p=top_p)
        got = B.spec_sample(to_dev(logits), to_dev(root), to_dev(toks), to_dev(q), to_dev(u), temperature=T,
                            select_mode=mode, has_root=has_root, prefix_len=100, top_p=top_p)
        assert got["status"] == 0
        total += 1
        if (_nucleus_margin(logits, root, has_root, n, k, T, top_p) <= 1e-12 or ref.commit_margin <= 1e-9 or
                (mode == 0 and min(ref.accept_margins.min(), ref.draw_margins.min()) <= 1e-9)):
            ties += 1
            continue
        np.testing.assert_array_equal(got["accept_len"], ref.accept_len)
        np.testing.assert_array_equal(got["next_token"], ref.next_token)
        assert (got["selected"], got["commit_len"], got["commit_token"], got["new_prefix_len"]) == \
               (ref.selected, ref.commit_len, ref.commit_token, ref.new_prefix_len)
    assert ties < total


def test_top_p_switched_off_values_change_nothing(B):
    logits, root, q, toks, u = _sampling_case(4099, 2, 4, 1, False, True)
    base = B.spec_sample(to_dev(logits), to_dev(root), to_dev(toks), to_dev(q), to_dev(u))
    for off in (1.0, 2.0, -0.5):
        got = B.spec_sample(to_dev(logits), to_dev(root), to_dev(toks), to_dev(q), to_dev(u), top_p=off)
        assert got["commit_token"] == base["commit_token"] and got["commit_len"] == base["commit_len"]
        np.testing.assert_array_equal(got["next_token"], base["next_token"])
    with pytest.raises(B.DuoError):
        B.spec_sample(to_dev(logits), to_dev(root), to_dev(toks), to_dev(q), to_dev(u), top_p=float("nan"))


def test_negative_temperature_is_rejected(B):
    logits, root, q, toks, u = _sampling_case(50, 1, 2, 0, False, False)
    with pytest.raises(B.DuoError):
        B.spec_sample(to_dev(logits), to_dev(root), to_dev(toks), to_dev(q), to_dev(u), temperature=-1.0)


def test_sampler_flags_out_of_range_token(B):
    logits, root, q, toks, u = _sampling_case(50, 1, 2, 0, False, False)
    toks[0, 1] = 50
    got = B.spec_sample(to_dev(logits), to_dev(root), to_dev(toks), to_dev(q), to_dev(u))
    assert got["status"] & B.STATUS_TOKEN_CLAMPED


# ------------------------------------------------------------------ the whole step
def _engine_and_oracle(B, shape, P, max_seq, seed, synthetic_cache, dtype="bf16", max_prefill_rows=80):
    w = inputs.make_weights(shape, seed=seed, threads=16, dtype=dtype)
    oshape = O.shape_from(shape)
    eng = B.VerifyEngine(shape, w, max_seq, max_prefill_rows=max_prefill_rows)
    assert eng.dtype == dtype
    if synthetic_cache:
        kb, vb, root = inputs.make_synthetic_cache(shape, P, max_seq, seed=seed, dtype=dtype)
        eng.load_cache(kb, vb, P, root)
        cache = O.OracleCache.from_bits(oshape, kb, vb, P, root)
        del kb, vb
    else:
        prefix = inputs.make_prefix_ids(shape, P, seed=seed)
        eng.prefill(prefix.tolist())
        cache = O.prefill(oshape, w, prefix.tolist(), max_seq)
    return w, oshape, eng, cache


def _check_step(B, shape, w, oshape, eng, cache, n, k, seed, mode, root_token, temperature=1.0):
    import torch
    V = shape.vocab
    q, toks, u = inputs.make_draft(V, n, k, seed=seed, easy_rows=inputs.easy_rows_for(n, k))
    R = 1 if root_token >= 0 else 0
    P = cache.prefix_len
    cache_root = None if cache.root_logits is None else cache.root_logits.copy()  # the oracle's commit drops it
    logits_dev = torch.empty((R + n * k, V), dtype=torch.float32, device="cuda")
    eng.verify(to_dev(toks), to_dev(q), to_dev(u), temperature=temperature, select_mode=mode, root_token=root_token,
               logits_out=logits_dev)
    got = eng.results(n)
    assert got["status"] == 0
    gl = logits_dev.cpu().numpy()
    res, ol = O.oracle_verify(oshape, w, cache, toks, q, u, temperature=temperature, select_mode=mode,
                              root_token=root_token)
    ok, max_abs, worst = logits_close(gl, ol)
    say(f"  logits max abs err {max_abs:.3e} (worst err/bound {worst:.3f}); gpu accept {got['accept_len']} "
        f"oracle {res.accept_len} accept margins {np.round(res.accept_margins, 4)}")
    assert ok, (max_abs, worst)
    # decisions, both modes: (1) bit-exact against the oracle's sampler on the logits the GPU returned; (2) against the
    # oracle's whole step on its own logits wherever its margins exceed the declared-tie bound
    groot = eng.root_logits.cpu().numpy()
    exact = same_as_sampler_on(got, gl, groot, toks, q, u, P, temperature, mode, bool(R))
    compared = compare_end_to_end(got, res, n, mode, ol, cache_root, q, u, k, R, temperature)
    say(f"  decisions: bit-exact on the GPU's logits {'compared' if exact else 'skipped (tie within 1e-9)'}; "
        f"{compared} compared against the oracle's own logits")
    # the fused call's sampler sees the same logits it returned: same decisions as the stand-alone sampler entry point
    again = B.spec_sample(logits_dev, eng.root_logits, to_dev(toks), to_dev(q), to_dev(u), temperature=temperature,
                          select_mode=mode, has_root=bool(R), prefix_len=P)
    for key in ("selected", "commit_len", "commit_token", "new_prefix_len"):
        assert again[key] == got[key], key
    np.testing.assert_array_equal(again["accept_len"], got["accept_len"])
    np.testing.assert_array_equal(again["next_token"], got["next_token"])
    assert got["new_prefix_len"] == P + R + got["commit_len"] == got["device_prefix_len"]
    return got, res, compared


def _check_cache(eng, cache, upto, atol=0.07):
    """GPU cache slots [0, upto) against the oracle's (bf16 values, a rounding flip is one ulp)."""
    kg, vg = eng.cache_to_host()
    kd = np.abs(O.bf16_bits_to_f64(kg[:, :, :upto]) - cache.k[:, :, :upto])
    vd = np.abs(O.bf16_bits_to_f64(vg[:, :, :upto]) - cache.v[:, :, :upto])
    say(f"  cache max abs diff k {kd.max():.3e} v {vd.max():.3e}")
    assert kd.max() <= atol and vd.max() <= atol


def _check_cache_rows(B, eng, cache, lo, hi, layers, atol=0.07):
    """Cache slots [lo, hi) of a few layers against the oracle's, moved to the host slot range only (full-size caches
    are gigabytes).  Returns the largest differences."""
    D = eng.shape.head_dim
    idx = list(layers)
    kg = B.k_tiles_to_rows(eng.k[idx], D)[:, :, lo:hi].cpu().numpy().view(np.uint16)
    vg = B.v_tiles_to_rows(eng.vT[idx], D)[:, :, lo:hi].cpu().numpy().view(np.uint16)
    kd = np.abs(O.bf16_bits_to_f64(kg) - cache.k[idx][:, :, lo:hi]).max() if hi > lo else 0.0
    vd = np.abs(O.bf16_bits_to_f64(vg) - cache.v[idx][:, :, lo:hi]).max() if hi > lo else 0.0
    assert kd <= atol and vd <= atol, (lo, hi, kd, vd)
    return kd, vd


def test_tiny_config_prefill_and_verify_chain(B):
    """68M-class shape: GPU prefill vs oracle prefill, then three chained verify steps with commits."""
    wl = inputs.WORKLOADS["C0"]
    shape, P = wl.shape, wl.prefix_len
    say("C0 prefill")
    w, oshape, eng, cache = _engine_and_oracle(B, shape, P, 256, seed=0, synthetic_cache=False)
    ok, max_abs, worst = logits_close(eng.root_logits.cpu().numpy(), cache.root_logits)
    say(f"  root logits max abs err {max_abs:.3e}")
    assert ok
    _check_cache(eng, cache, P)
    root = -1
    for step, (n, k, mode) in enumerate([(1, 8, 0), (3, 5, 1), (4, 8, 0)]):
        say(f"C0 step {step}: n={n} k={k} mode={mode} root={root} P={cache.prefix_len}")
        got, res, _ = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=10 + step, mode=mode, root_token=root)
        same = (got["selected"], got["commit_len"]) == (res.selected, res.commit_len)
        if not same:  # a declared tie moved the commit: put both sides on the oracle's state
            say("  commit differs (declared tie); stopping the chain")
            break
        _check_cache(eng, cache, cache.prefix_len)
        root = res.commit_token


@pytest.mark.parametrize("n,k,mode,root", [(3, 5, 1, 17), (1, 16, 0, -1), (4, 16, 0, 3), (8, 8, 1, -1), (2, 1, 0, 5),
                                            (3, 8, 0, -1), (2, 16, 1, 9), (5, 8, 0, -1), (1, 9, 0, -1), (5, 16, 0, -1),
                                            (1, 1, 0, -1), (7, 7, 0, 3), (6, 8, 1, -1)])
def test_mid_config_gqa_ragged(B, n, k, mode, root):
    """3 layers, 8 query / 2 KV heads of 64, vocab 4099 (not a multiple of 16), prefix 77.  The row counts
    (16, 16, 65, 64, 3, 24, 33, 40, 9, 80, 1, 50, 48) cover every row-tile count of both projection kernels, the
    largest call the library takes (80 rows), the smallest (one token) and both sides of the row count from which the
    Q/K/V projection splits K over workgroups (49)."""
    shape = inputs.MID
    say(f"MID n={n} k={k} mode={mode} root={root}")
    w, oshape, eng, cache = _engine_and_oracle(B, shape, 77, 192, seed=2, synthetic_cache=False)
    got, res, _ = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=n * 31 + k, mode=mode, root_token=root)
    if (got["selected"], got["commit_len"]) == (res.selected, res.commit_len):
        _check_cache(eng, cache, cache.prefix_len)


@pytest.mark.parametrize("n,k,root,P", [(1, 8, -1, 1100), (2, 8, -1, 1100), (1, 3, 7, 1100), (2, 6, 4, 1371), (1, 5, -1, 2045),
                                        (8, 8, -1, 1100), (7, 7, 3, 1371), (5, 16, -1, 2045), (4, 16, -1, 1056)])
def test_mid_config_long_prefix(B, n, k, root, P):
    """The MID shape (GQA group of 4, heads of 64) on a long synthetic prefix, so that a head's keys are cut into
    several chunks: 32, 64, 16, 52 and 20 (row, query head) pairs per KV head = 2, 4, 1, 4 and 2 query tiles, i.e. the
    attention kernel whose waves form two teams over the key blocks (two and four tiles per workgroup, chunks of an even
    and an odd number of blocks, a last block that is partly draft slots) and, for one tile, the per-wave kernel; the
    chunk merge in all of them.  The cases of 64, 50, 80 and 64 rows add the K-split Q/K/V projection with its finish
    kernel and 16 to 20 query tiles per KV head: prefixes that end inside a 32-key block and on a block boundary, with
    and without a root row, sequences of 7, 8 and 16 tokens."""
    shape = inputs.MID
    say(f"MID long prefix P={P} n={n} k={k} root={root}")
    max_seq = (P + 1 + n * k + 31) // 32 * 32
    w, oshape, eng, cache = _engine_and_oracle(B, shape, P, max_seq, seed=5, synthetic_cache=True)
    got, res, _ = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=n * 17 + k, mode=0, root_token=root)
    if (got["selected"], got["commit_len"]) == (res.selected, res.commit_len):
        _check_cache_rows(B, eng, cache, P, cache.prefix_len, range(shape.n_layers))


@pytest.mark.parametrize("n,k,root,P", [(7, 7, -1, 40), (8, 8, 5, 64), (5, 16, -1, 1)])
def test_mid_config_many_rows_short_prefix(B, n, k, root, P):
    """49, 65 and 80 rows (the K-split Q/K/V projection) on a prefix of at most two key blocks: one key chunk per head,
    draft slots in every block."""
    shape = inputs.MID
    say(f"MID short prefix P={P} n={n} k={k} root={root}")
    w, oshape, eng, cache = _engine_and_oracle(B, shape, P, 160, seed=9, synthetic_cache=False)
    got, res, _ = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=n * 13 + k, mode=0, root_token=root)
    if (got["selected"], got["commit_len"]) == (res.selected, res.commit_len):
        _check_cache(eng, cache, cache.prefix_len)


@pytest.mark.parametrize("mode,root", [(0, -1), (1, 12)])
def test_mid_config_greedy_step(B, mode, root):
    """A whole step at temperature 0.  The logits are compared as always; the decisions are the arg-max rule applied to
    the logits the GPU returned (an arg max taken on the oracle's own logits could differ at near-equal logits)."""
    import torch
    shape = inputs.MID
    n, k = 3, 5
    say(f"MID greedy mode={mode} root={root}")
    w, oshape, eng, cache = _engine_and_oracle(B, shape, 77, 192, seed=2, synthetic_cache=False)
    q, toks, u = inputs.make_draft(shape.vocab, n, k, seed=5)
    # make the drafts follow the oracle's arg max for a while, so that accepted lengths are not all zero
    ol = O.verify_forward(oshape, w, cache, toks, root).astype(np.float32)  # the forward pass alone commits nothing
    R = 1 if root >= 0 else 0
    toks[1, 0] = int(np.argmax(ol[0] if R else cache.root_logits))
    ol = O.verify_forward(oshape, w, cache, toks, root).astype(np.float32)
    toks[1, 1] = int(np.argmax(ol[R + k]))
    lg = torch.empty((R + n * k, shape.vocab), dtype=torch.float32, device="cuda")
    eng.verify(to_dev(toks), to_dev(q), to_dev(u), temperature=0.0, select_mode=mode, root_token=root, logits_out=lg)
    got = eng.results(n)
    assert got["status"] == 0
    gl = lg.cpu().numpy()
    ol = O.verify_forward(oshape, w, cache, toks, root).astype(np.float32)
    ok, max_abs, worst = logits_close(gl, ol)
    assert ok, (max_abs, worst)
    ref = O.speculative_verify(gl, eng.root_logits.cpu().numpy(), toks, q, u, prefix_len=77, temperature=0.0,
                               select_mode=mode, has_root=bool(R))
    say(f"  gpu accept {got['accept_len']} commit {got['selected']}/{got['commit_len']}/{got['commit_token']}")
    np.testing.assert_array_equal(got["accept_len"], ref.accept_len)
    np.testing.assert_array_equal(got["next_token"], ref.next_token)
    assert (got["selected"], got["commit_len"], got["commit_token"], got["new_prefix_len"]) == \
           (ref.selected, ref.commit_len, ref.commit_token, ref.new_prefix_len)
    assert got["commit_len"] >= 1


@pytest.mark.parametrize("chunks", [(300,), (200, 130), (81, 512), (1024,), (40, 95)])
def test_many_row_prefill_matches_oracle(B, chunks):
    """Prompt chunks of more than 80 rows run through the block projection kernel (K-split residual projections at
    this width): root logits and cache against the oracle's prefill, then one verify step on top."""
    shape = inputs.MID
    total = sum(chunks)
    max_seq = (total + 40 + 31) // 32 * 32
    say(f"MID many-row prefill chunks={chunks}")
    w = inputs.make_weights(shape, seed=4, threads=16)
    oshape = O.shape_from(shape)
    eng = B.VerifyEngine(shape, w, max_seq, max_prefill_rows=max(chunks))
    prefix = inputs.make_prefix_ids(shape, total, seed=4)
    at = 0
    for c in chunks:
        eng.prefill(prefix[at:at + c].tolist(), chunk=c)
        at += c
    cache = O.prefill(oshape, w, prefix.tolist(), max_seq)
    ok, max_abs, worst = logits_close(eng.root_logits.cpu().numpy(), cache.root_logits)
    say(f"  root logits max abs err {max_abs:.3e} (worst err/bound {worst:.3f})")
    assert ok
    _check_cache(eng, cache, total)
    assert int(eng.prefix_len.item()) == total
    _check_step(B, shape, w, oshape, eng, cache, 2, 4, seed=9, mode=0, root_token=-1)


def test_many_row_prefill_full_width_layer(B):
    """One layer of 7B width, 1007 prompt rows: the launch shapes of a full-size chunk (unsplit residual projections
    with the residual epilogue in the block kernel, the wider blocks for QKV and gate/up, heads of 128, GQA)."""
    shape = inputs.WIDE1
    total = 1007
    max_seq = 1056
    say("WIDE1 many-row prefill 1007 rows")
    w = inputs.make_weights(shape, seed=6, threads=16)
    oshape = O.shape_from(shape)
    eng = B.VerifyEngine(shape, w, max_seq, max_prefill_rows=total)
    prefix = inputs.make_prefix_ids(shape, total, seed=6)
    eng.prefill(prefix.tolist(), chunk=total)
    cache = O.prefill(oshape, w, prefix.tolist(), max_seq)
    ok, max_abs, worst = logits_close(eng.root_logits.cpu().numpy(), cache.root_logits)
    say(f"  root logits max abs err {max_abs:.3e} (worst err/bound {worst:.3f})")
    assert ok
    _check_cache(eng, cache, total)


@pytest.mark.parametrize("n,k,mode", [(2, 4, 0), (1, 1, 0), (3, 5, 1)])
def test_empty_prefix_with_root_token(B, n, k, mode):
    """Nothing cached yet: the root token is the first token of the text (position 0) and the only shared context."""
    shape = inputs.MID
    say(f"MID empty prefix n={n} k={k} mode={mode}")
    w, oshape, eng, cache = _engine_and_oracle(B, shape, 0, 64, seed=11, synthetic_cache=True)
    assert cache.prefix_len == 0
    got, res, _ = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=4, mode=mode, root_token=9)
    assert got["new_prefix_len"] == 1 + got["commit_len"]
    if (got["selected"], got["commit_len"]) == (res.selected, res.commit_len):
        _check_cache(eng, cache, cache.prefix_len)


@pytest.mark.parametrize("n,k,root", [(1, 8, -1), (4, 16, 3), (2, 12, -1)])
def test_other_width_single_layer(B, n, k, root):
    """One layer of 13B width: the launch rules (waves per band group, K splits, attention shapes) at band counts
    and K ranges other than those of the benchmark shapes."""
    shape = inputs.WIDE13
    say(f"WIDE13 n={n} k={k} root={root}")
    w, oshape, eng, cache = _engine_and_oracle(B, shape, 300, 448, seed=13, synthetic_cache=True)
    got, res, _ = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=n + k, mode=0, root_token=root)
    if (got["selected"], got["commit_len"]) == (res.selected, res.commit_len):
        _check_cache(eng, cache, cache.prefix_len)


@pytest.mark.parametrize("n,k,root", [(1, 8, -1), (1, 7, 5), (4, 8, -1), (5, 16, -1), (2, 3, -1), (7, 7, -1), (8, 8, 11)])
def test_7b_width_single_layer(B, n, k, root):
    """One layer of 7B width: the launch shapes of the benchmark step (768 independent Q/K/V bands, one per wave up to
    80 rows; gate/up and down at d_ff 11008) at 6, 8, 32 and 80 rows."""
    shape = inputs.WIDE7
    say(f"WIDE7 n={n} k={k} root={root}")
    w, oshape, eng, cache = _engine_and_oracle(B, shape, 300, 448, seed=17, synthetic_cache=True)
    got, res, _ = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=2 * n + k, mode=0, root_token=root)
    if (got["selected"], got["commit_len"]) == (res.selected, res.commit_len):
        _check_cache(eng, cache, cache.prefix_len)


@pytest.mark.parametrize("mode,root,top_p", [(0, -1, 0.8), (1, 12, 0.5), (0, 3, 0.95)])
def test_mid_config_top_p_step(B, mode, root, top_p):
    """A whole step with nucleus sampling: logits against the oracle's forward pass, decisions against the oracle's
    sampler applied to the logits the GPU returned (the nucleus of slightly different logits can differ)."""
    import torch
    shape = inputs.MID
    n, k = 3, 5
    say(f"MID top-p step mode={mode} root={root} top_p={top_p}")
    w, oshape, eng, cache = _engine_and_oracle(B, shape, 77, 192, seed=2, synthetic_cache=False)
    q, toks, u = inputs.make_draft(shape.vocab, n, k, seed=6, easy_rows=inputs.easy_rows_for(n, k))
    R = 1 if root >= 0 else 0
    lg = torch.empty((R + n * k, shape.vocab), dtype=torch.float32, device="cuda")
    eng.verify(to_dev(toks), to_dev(q), to_dev(u), temperature=0.9, select_mode=mode, root_token=root, logits_out=lg,
               top_p=top_p)
    got = eng.results(n)
    assert got["status"] == 0
    gl = lg.cpu().numpy()
    ol = O.verify_forward(oshape, w, cache, toks, root).astype(np.float32)
    ok, max_abs, worst = logits_close(gl, ol)
    assert ok, (max_abs, worst)
    groot = eng.root_logits.cpu().numpy()
    ref = O.speculative_verify(gl, groot, toks, q, u, prefix_len=77, temperature=0.9, select_mode=mode, has_root=bool(R),
                               top_p=top_p)
    say(f"  gpu accept {got['accept_len']} commit {got['selected']}/{got['commit_len']}/{got['commit_token']}")
    if (_nucleus_margin(gl, groot, bool(R), n, k, 0.9, top_p) <= 1e-12 or ref.commit_margin <= 1e-9 or
            (mode == 0 and min(ref.accept_margins.min(), ref.draw_margins.min()) <= 1e-9)):
        pytest.skip("a decision within rounding of a tie")
    np.testing.assert_array_equal(got["accept_len"], ref.accept_len)
    np.testing.assert_array_equal(got["next_token"], ref.next_token)
    assert (got["selected"], got["commit_len"], got["commit_token"], got["new_prefix_len"]) == \
           (ref.selected, ref.commit_len, ref.commit_token, ref.new_prefix_len)


def test_cache_filled_to_the_last_slot(B):
    """prefix + rows == max_seq exactly: the last cache slot is written and read; one more row is refused."""
    shape = inputs.MID
    n, k, P = 2, 8, 48  # 16 rows, cache of 64 slots
    w, oshape, eng, cache = _engine_and_oracle(B, shape, P, P + n * k, seed=7, synthetic_cache=True)
    got, res, _ = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=3, mode=0, root_token=-1)
    if (got["selected"], got["commit_len"]) == (res.selected, res.commit_len):
        _check_cache(eng, cache, cache.prefix_len)
    eng.set_prefix_len(P)
    q, toks, u = inputs.make_draft(shape.vocab, n, k, seed=3)
    with pytest.raises(B.DuoError):  # 48 + 1 + 16 rows do not fit 64 slots
        eng.verify(to_dev(toks), to_dev(q), to_dev(u), root_token=5)


def test_verify_is_repeatable_and_flags_prefix_mismatch(B):
    import torch
    shape = inputs.MID
    w, oshape, eng, cache = _engine_and_oracle(B, shape, 40, 128, seed=5, synthetic_cache=True)
    q, toks, u = inputs.make_draft(shape.vocab, 2, 4, seed=1)
    outs = []
    for rep in range(2):
        eng.set_prefix_len(40)
        lg = torch.empty((8, shape.vocab), dtype=torch.float32, device="cuda")
        eng.verify(to_dev(toks), to_dev(q), to_dev(u), logits_out=lg)
        r = eng.results(2)
        outs.append((lg.cpu().numpy(), r))
    np.testing.assert_array_equal(outs[0][0], outs[1][0])  # bit-identical: no atomics in any reduction
    assert outs[0][1]["commit_token"] == outs[1][1]["commit_token"]
    eng.host_prefix_len = 41  # host and device now disagree
    eng.verify(to_dev(toks), to_dev(q), to_dev(u))
    assert eng.results(2)["status"] & B.STATUS_PREFIX_MISMATCH


def test_device_detected_failures_commit_nothing(B):
    """A call that fails on the device (stale host prefix length, draft token out of range) is flagged and leaves the
    prefix length, the root logits and every committed cache slot exactly as they were; the next good call gives
    what it gave before."""
    import torch
    shape = inputs.MID
    P, max_seq = 40, 128
    w, oshape, eng, cache = _engine_and_oracle(B, shape, P, max_seq, seed=5, synthetic_cache=True)
    q, toks, u = inputs.make_draft(shape.vocab, 2, 4, seed=1)
    d = [to_dev(a) for a in (toks, q, u)]

    def committed_state():
        torch.cuda.synchronize()
        kc, vc = eng.cache_to_host()
        return kc[:, :, :P].copy(), vc[:, :, :P].copy(), int(eng.prefix_len.item()), eng.root_logits.cpu().numpy().copy()

    def unchanged(before):
        now = committed_state()
        np.testing.assert_array_equal(now[0], before[0])
        np.testing.assert_array_equal(now[1], before[1])
        assert now[2] == before[2] == P
        np.testing.assert_array_equal(now[3], before[3])

    eng.verify(*d)
    good = eng.results(2)
    assert good["status"] == 0 and good["new_prefix_len"] == P + good["commit_len"]
    eng.set_prefix_len(P)
    before = committed_state()
    for mode in (0, 1):
        for stale in (33, 44):  # too small: the pass's rows would land on committed slots; too large: a hole
            say(f"failure: host prefix {stale}, device prefix {P}, mode {mode}")
            eng.host_prefix_len = stale
            eng.verify(*d, select_mode=mode)
            r = eng.results(2)
            assert r["status"] & B.STATUS_PREFIX_MISMATCH
            assert (r["selected"], r["commit_len"], r["commit_token"], r["new_prefix_len"]) == (-1, 0, -1, P)
            assert eng.host_prefix_len == P  # the commit record reports the device's prefix length
            unchanged(before)
        say(f"failure: draft token out of range, mode {mode}")
        bad = toks.copy()
        bad[1, 2] = shape.vocab + 5
        eng.verify(to_dev(bad), d[1], d[2], select_mode=mode)
        r = eng.results(2)
        assert r["status"] & B.STATUS_TOKEN_CLAMPED
        assert (r["selected"], r["commit_len"], r["commit_token"], r["new_prefix_len"]) == (-1, 0, -1, P)
        unchanged(before)
    say("failure: single-sequence call (the sampler commits itself), deferred form, prompt chunk")
    eng.host_prefix_len = 37
    eng.verify(d[0][:1], d[1][:1], d[2][:1])
    r = eng.results(1)
    assert r["status"] & B.STATUS_PREFIX_MISMATCH and r["new_prefix_len"] == P and r["commit_len"] == 0
    unchanged(before)
    eng.host_prefix_len = 37
    eng.verify_deferred(d[0][0], d[1][0], d[2][0], d[0][:, 0].contiguous(), d[1][:, 0].contiguous(), d[2][:, 0].contiguous(), root_token=3)
    r = eng.results(1)
    assert r["status"] & B.STATUS_PREFIX_MISMATCH and r["new_prefix_len"] == P and r["selected"] == -1
    unchanged(before)
    eng.host_prefix_len = 36
    eng.prefill([1, 2, 3, 4, 5])  # a stale host: the chunk must not become part of the prefix
    torch.cuda.synchronize()
    assert int(eng.status.item()) & B.STATUS_PREFIX_MISMATCH
    unchanged(before)
    eng.host_prefix_len = P
    eng.verify(*d)
    again = eng.results(2)
    assert again["status"] == 0
    for key in ("selected", "commit_len", "commit_token", "new_prefix_len"):
        assert again[key] == good[key], key
    np.testing.assert_array_equal(again["accept_len"], good["accept_len"])


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4"])
def test_full_size_shapes(B, name):
    """Llama-2-7B (C1-C3) and Llama-3-8B GQA (C4) geometry at the benchmark's launch configuration, synthetic
    prefix cache: every logit of every row against the oracle, accept lengths away from ties."""
    wl = inputs.WORKLOADS[name]
    shape, P, n, k = wl.shape, wl.prefix_len, wl.n_seq, wl.k_draft
    say(f"{name}: generating weights")
    w, oshape, eng, cache = _engine_and_oracle(B, shape, P, P + 128, seed=0, synthetic_cache=True)
    say(f"{name}: verify n={n} k={k} P={P}")
    root0 = cache.root_logits.copy()
    got, res, compared = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=1, mode=0, root_token=-1)
    say(f"  accept lengths compared away from ties: {compared}/{n}")
    assert 2 * compared >= n
    # the commit at full size: the selected branch's keys and values next to the prefix (first, middle and last layer),
    # the prefix itself untouched (bit-identical to what was loaded), the prefix length advanced on the device
    layers = sorted({0, shape.n_layers // 2, shape.n_layers - 1})
    assert (got["selected"], got["commit_len"]) == (res.selected, res.commit_len), "no declared tie on these inputs"
    assert cache.prefix_len == P + res.commit_len == got["device_prefix_len"]
    kd, vd = _check_cache_rows(B, eng, cache, P, cache.prefix_len, layers)
    _check_cache_rows(B, eng, cache, 0, 64, layers, atol=0.0)
    _check_cache_rows(B, eng, cache, P - 64, P, layers, atol=0.0)
    say(f"  committed rows [{P}, {cache.prefix_len}) of layers {layers}: max abs diff k {kd:.3e} v {vd:.3e}; prefix rows identical")
    if n > 1:  # and the multi-sequence rule of Alg. 2 on the same state
        eng.set_prefix_len(P)
        cache.prefix_len = P
        cache.root_logits = root0
        say(f"{name}: the same step in paper mode")
        got, res, compared = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=1, mode=1, root_token=-1)
        assert compared >= 1


def test_full_size_prefill_paths_agree(B):
    """Llama-2-7B geometry, 1100 prompt tokens: the many-row pass (one chunk of 1024 rows and one of 76) against the
    few-row pass (chunks of 80 rows) of the same library.  At this size the oracle would take an hour; each pass is
    checked against it at small sizes above, here they must agree with each other: last-row logits within twice the
    logit tolerance, cached keys and values within one bf16 rounding step of values of this size."""
    import torch
    shape = inputs.LLAMA2_7B
    total = 1100
    say("7B prefill: generating weights")
    w = inputs.make_weights(shape, seed=0, threads=16)
    dw = B.DeviceWeights(shape, w)
    prompt = inputs.make_prefix_ids(shape, total, seed=3).tolist()
    outs = []
    for chunk in (1024, 80):
        say(f"7B prefill in chunks of {chunk}")
        eng = B.VerifyEngine(shape, None, 1152, weights=dw, max_prefill_rows=chunk)
        eng.prefill(prompt, chunk=chunk)
        torch.cuda.synchronize()
        assert int(eng.prefix_len.item()) == total and int(eng.status.item()) == 0
        kc, vc = eng.cache_to_host()
        outs.append((eng.root_logits.cpu().numpy().copy(), O.bf16_bits_to_f64(kc[::8, :, :total]), O.bf16_bits_to_f64(vc[::8, :, :total])))
        # What the oracle can compute one by one at this size: the first layer's keys and values of sampled prompt
        # positions depend on their own token only (embedding, RMSNorm, the K/V projections, the rotation at the
        # token's position), so they are checked against the oracle's pieces directly, through both row paths.
        for t in (0, 1, 79, 80, 511, 1023, 1024, total - 1):
            x = O.embed_rows(w, [prompt[t]])
            h = O.rmsnorm(x, O._w(w, "g_attn", 0), shape.rms_eps)
            k_ref = (h @ O._w(w, "wk", 0).T).reshape(shape.n_kv_heads, shape.head_dim)
            k_ref = O.round_to_bf16(np.stack([O.rope(k_ref[a], t, shape.rope_theta) for a in range(shape.n_kv_heads)]))
            v_ref = O.round_to_bf16((h @ O._w(w, "wv", 0).T).reshape(shape.n_kv_heads, shape.head_dim))
            dk = np.abs(O.bf16_bits_to_f64(kc[0, :, t]) - k_ref).max()
            dv = np.abs(O.bf16_bits_to_f64(vc[0, :, t]) - v_ref).max()
            assert dk <= 0.07 and dv <= 0.07, (chunk, t, dk, dv)   # one bf16 step at values of this size
            assert np.abs(k_ref).max() > 0.5
        del eng
    (la, ka, va), (lb, kb, vb) = outs
    dl = np.abs(la - lb)
    say(f"  last-row logits max abs diff {dl.max():.3e}; cache max abs diff k {np.abs(ka - kb).max():.3e} v {np.abs(va - vb).max():.3e}")
    assert (dl <= 2 * (2e-2 + 1e-2 * np.abs(lb))).all()
    assert np.abs(ka - kb).max() <= 0.07 and np.abs(va - vb).max() <= 0.07
    assert np.abs(ka).max() > 0.5 and np.abs(la).max() > 0.5   # not comparing zeros


# ------------------------------------------------------------------ the fp16 build (the same sources, DUO_FP16)
@pytest.mark.parametrize("rows,N,K", [(8, 4096, 4096), (33, 4099, 1408), (80, 515, 96)])
def test_fp16_skinny_gemm_matches_oracle_matmul(B, rows, N, K):
    import torch
    say(f"fp16 gemm rows={rows} N={N} K={K}")
    g = np.random.default_rng(rows * 1000 + N)
    x = g.normal(0, 1, (rows, K)).astype(np.float16)
    w = g.normal(0, 0.02, (N, K)).astype(np.float16)
    y = B.skinny_gemm(to_dev(x.view(np.int16)), to_dev(w.view(np.int16)), dtype="fp16")
    torch.cuda.synchronize()
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    err = np.abs(y.cpu().numpy() - ref).max()
    say(f"  max abs err {err:.3e}")
    assert err <= 2e-6 * np.sqrt(K) * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("rows,N,K", [(128, 4096, 4096), (300, 4099, 1408)])
def test_fp16_block_gemm_matches_oracle_matmul(B, rows, N, K):
    import torch
    say(f"fp16 block gemm rows={rows} N={N} K={K}")
    g = np.random.default_rng(rows * 1000 + N)
    a = g.normal(0, 1, (rows, K)).astype(np.float32)
    hi = a.astype(np.float16)
    lo = (a.astype(np.float64) - hi.astype(np.float64)).astype(np.float16)
    w = g.normal(0, 0.02, (N, K)).astype(np.float16)
    y = B.block_gemm(to_dev(hi.view(np.int16)), to_dev(lo.view(np.int16)), to_dev(w.view(np.int16)), dtype="fp16")
    torch.cuda.synchronize()
    ref = (hi.astype(np.float64) + lo.astype(np.float64)) @ w.astype(np.float64).T
    err = np.abs(y.cpu().numpy() - ref).max()
    say(f"  max abs err {err:.3e}")
    assert err <= 2e-6 * np.sqrt(K) * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("n,k,mode,root", [(1, 8, 0, -1), (3, 5, 1, 17), (5, 16, 0, -1), (4, 8, 0, 3)])
def test_fp16_mid_config_step(B, n, k, mode, root):
    """fp16 parameters and KV cache (the paper's precision): prefill and one verify step against the oracle run on the
    same float16 parameters, same tolerance as the bf16 build."""
    shape = inputs.MID
    say(f"fp16 MID n={n} k={k} mode={mode} root={root}")
    w, oshape, eng, cache = _engine_and_oracle(B, shape, 77, 192, seed=2, synthetic_cache=False, dtype="fp16")
    ok, max_abs, worst = logits_close(eng.root_logits.cpu().numpy(), cache.root_logits)
    assert ok
    _check_cache(eng, cache, 77, atol=0.01)   # fp16 cache: a rounding flip is 8x smaller than in bf16
    got, res, _ = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=n * 31 + k, mode=mode, root_token=root)
    if (got["selected"], got["commit_len"]) == (res.selected, res.commit_len):
        _check_cache(eng, cache, cache.prefix_len, atol=0.01)


def test_fp16_many_row_prefill(B):
    shape = inputs.MID
    chunks = (300, 95)
    total = sum(chunks)
    say("fp16 MID many-row prefill")
    w = inputs.make_weights(shape, seed=4, threads=16, dtype="fp16")
    oshape = O.shape_from(shape)
    eng = B.VerifyEngine(shape, w, 448, max_prefill_rows=max(chunks))
    prefix = inputs.make_prefix_ids(shape, total, seed=4)
    at = 0
    for c in chunks:
        eng.prefill(prefix[at:at + c].tolist(), chunk=c)
        at += c
    cache = O.prefill(oshape, w, prefix.tolist(), 448)
    ok, max_abs, worst = logits_close(eng.root_logits.cpu().numpy(), cache.root_logits)
    say(f"  root logits max abs err {max_abs:.3e}")
    assert ok
    _check_cache(eng, cache, total, atol=0.01)


def test_fp16_full_size_shape(B):
    """Llama-2-7B geometry in fp16 at the benchmark's launch configuration (C1)."""
    wl = inputs.WORKLOADS["C1"]
    shape, P, n, k = wl.shape, wl.prefix_len, wl.n_seq, wl.k_draft
    say("fp16 C1: generating weights")
    w, oshape, eng, cache = _engine_and_oracle(B, shape, P, P + 128, seed=0, synthetic_cache=True, dtype="fp16")
    got, res, compared = _check_step(B, shape, w, oshape, eng, cache, n, k, seed=1, mode=0, root_token=-1)
