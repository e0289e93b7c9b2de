"""Pins for the oracle's target pass: library model, brute force, invariants, closed forms."""
import numpy as np
import pytest

from oracle import duo_oracle as O


def tiny_shape(**kw):
    base = dict(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ff=48, vocab=50,
                rope_theta=10000.0, rms_eps=1e-5)
    base.update(kw)
    return O.OracleShape(**base)


def float_weights(shape, seed=0, scale=0.3):
    """Float64 weights (not bf16) with distinct, non-symmetric values."""
    g = np.random.default_rng(seed)
    d, f = shape.d_model, shape.d_ff
    qd, kd = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    L = shape.n_layers
    w = {
        "embed": g.normal(0, 1.0, (shape.vocab, d)),
        "lm_head": g.normal(0, scale, (shape.vocab, d)),
        "g_final": 1 + g.normal(0, 0.2, d),
        "wq": [g.normal(0, scale, (qd, d)) for _ in range(L)],
        "wk": [g.normal(0, scale, (kd, d)) for _ in range(L)],
        "wv": [g.normal(0, scale, (kd, d)) for _ in range(L)],
        "wo": [g.normal(0, scale, (d, qd)) for _ in range(L)],
        "w_gate": [g.normal(0, scale, (f, d)) for _ in range(L)],
        "w_up": [g.normal(0, scale, (f, d)) for _ in range(L)],
        "w_down": [g.normal(0, scale, (d, f)) for _ in range(L)],
        "g_attn": [1 + g.normal(0, 0.2, d) for _ in range(L)],
        "g_ffn": [1 + g.normal(0, 0.2, d) for _ in range(L)],
    }
    return w


# ------------------------------------------------------------------ closed forms of the pieces
def test_rmsnorm_closed_form_and_scale_invariance():
    g = np.array([1.0, 2.0, -0.5, 3.0])
    x = np.full(4, 3.0)
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-5), g * 3.0 / np.sqrt(9.0 + 1e-5), rtol=1e-15)
    x = np.array([3.0, -4.0, 0.0, 0.0])  # mean square = 25/4
    np.testing.assert_allclose(O.rmsnorm(x, np.ones(4), 0.0), x / 2.5, rtol=1e-15)
    y = np.random.default_rng(0).normal(size=16)
    np.testing.assert_allclose(O.rmsnorm(7.0 * y, np.ones(16), 0.0), O.rmsnorm(y, np.ones(16), 0.0), rtol=1e-13)


def test_rope_hand_values():
    # D = 2: a single pair rotated by pos * theta^0 = pos radians
    np.testing.assert_allclose(O.rope(np.array([1.0, 0.0]), 3, 10000.0), [np.cos(3.0), np.sin(3.0)], rtol=1e-15)
    # D = 4, theta = 100: pair (0,2) turns by pos, pair (1,3) by pos * 100^(-1/2) = pos / 10
    v = np.array([1.0, 2.0, 3.0, 4.0])
    out = O.rope(v, 5, 100.0)
    a0, a1 = 5.0, 0.5
    exp = [1 * np.cos(a0) - 3 * np.sin(a0), 2 * np.cos(a1) - 4 * np.sin(a1),
           3 * np.cos(a0) + 1 * np.sin(a0), 4 * np.cos(a1) + 2 * np.sin(a1)]
    np.testing.assert_allclose(out, exp, rtol=1e-14)
    np.testing.assert_array_equal(O.rope(v, 0, 100.0), v)


def test_rope_relative_shift_and_norm():
    g = np.random.default_rng(1)
    q, k = g.normal(size=16), g.normal(size=16)
    d1 = O.rope(q, 17, 10000.0) @ O.rope(k, 11, 10000.0)
    d2 = O.rope(q, 1017, 10000.0) @ O.rope(k, 1011, 10000.0)
    assert abs(d1 - d2) < 1e-10
    assert abs(np.linalg.norm(O.rope(q, 123, 10000.0)) - np.linalg.norm(q)) < 1e-12


def test_silu_and_softmax_values():
    assert abs(O.silu(np.array(1.0)) - 0.7310585786300049) < 1e-15
    assert abs(O.silu(np.array(-2.0)) - (-2.0 / (1 + np.exp(2.0)))) < 1e-15
    s = O.softmax(np.array([np.log(1.0), np.log(2.0), np.log(5.0)]))
    np.testing.assert_allclose(s, [0.125, 0.25, 0.625], rtol=1e-14)
    np.testing.assert_allclose(O.softmax(np.array([1000.0, 1000.0])), [0.5, 0.5])


def test_bf16_rounding_ties_to_even_and_matches_torch():
    import torch
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0              # tie -> even mantissa
    assert O.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    x = np.random.default_rng(0).normal(size=4096).astype(np.float32)
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_to_bf16(x), t)
    bits = O.f64_to_bf16_bits(x)
    np.testing.assert_array_equal(O.bf16_bits_to_f64(bits), t)


def test_generator_bf16_packing_matches_torch():
    import torch
    from paper_2503_00784_amd import inputs
    x = np.random.default_rng(3).normal(size=5000).astype(np.float32)
    bits = inputs.f32_to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, t)


# ------------------------------------------------------------------ the library the paper builds on
@pytest.mark.parametrize("hq,hkv", [(4, 2), (4, 4)])
def test_forward_matches_hf_transformers_llama(hq, hkv):
    torch = pytest.importorskip("torch")
    tr = pytest.importorskip("transformers")
    shape = tiny_shape(n_q_heads=hq, n_kv_heads=hkv)
    w = float_weights(shape, seed=5)
    cfg = tr.LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ff,
                         num_hidden_layers=shape.n_layers, num_attention_heads=hq, num_key_value_heads=hkv,
                         head_dim=shape.head_dim, rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_theta,
                         max_position_embeddings=64, tie_word_embeddings=False, attention_bias=False,
                         mlp_bias=False, hidden_act="silu")
    model = tr.LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "model.norm.weight": w["g_final"], "lm_head.weight": w["lm_head"]}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj", "wo": "self_attn.o_proj",
             "w_gate": "mlp.gate_proj", "w_up": "mlp.up_proj", "w_down": "mlp.down_proj",
             "g_attn": "input_layernorm", "g_ffn": "post_attention_layernorm"}
    for key, hf in names.items():
        for l in range(shape.n_layers):
            sd[f"model.layers.{l}.{hf}.weight"] = w[key][l]
    missing = model.load_state_dict({k: torch.from_numpy(np.asarray(v)) for k, v in sd.items()}, strict=False)
    assert not [m for m in missing.missing_keys if "rotary" not in m]
    tokens = [3, 17, 42, 8, 8, 29, 0, 49, 11]
    with torch.no_grad():
        ref = model(torch.tensor([tokens])).logits[0].numpy()
    got = O.full_forward_uncached(shape, w, tokens, rounding="ideal")
    # the library keeps its rotary cos/sin tables in float32 even for a float64 model, which
    # limits the agreement to ~1e-6; a wrong convention anywhere gives O(1) differences
    np.testing.assert_allclose(got, ref, rtol=1e-5, atol=5e-6)
    # cached, row-by-row pass: prefix of 5, then one draft sequence of 4
    cache = O.prefill(shape, w, tokens[:5], max_seq=16, rounding="ideal")
    np.testing.assert_allclose(cache.root_logits, ref[4].astype(np.float32), rtol=1e-5, atol=5e-6)
    lg = O.verify_forward(shape, w, cache, np.array([tokens[5:]]), rounding="ideal")
    np.testing.assert_allclose(lg, ref[5:], rtol=1e-5, atol=5e-6)
    np.testing.assert_allclose(lg, got[5:], rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------ structure of the method
def _setup(seed=0, P=6, max_seq=40, **kw):
    shape = tiny_shape(**kw)
    w = float_weights(shape, seed=seed)
    g = np.random.default_rng(seed + 100)
    prefix = g.integers(0, shape.vocab, P).tolist()
    cache = O.prefill(shape, w, prefix, max_seq=max_seq, rounding="ideal")
    return shape, w, prefix, cache, g


def test_parallel_pass_equals_sequential_single_token_decodes():
    shape, w, prefix, cache, g = _setup()
    drafts = g.integers(0, shape.vocab, (1, 5))
    par = O.verify_forward(shape, w, cache.copy(), drafts, rounding="ideal")
    c = cache.copy()
    for j in range(5):
        step = O.verify_forward(shape, w, c, drafts[:, j:j + 1], rounding="ideal")
        np.testing.assert_allclose(step[0], par[j], rtol=1e-10, atol=1e-12)
        c.prefix_len += 1  # the token just scored becomes part of the prefix


def test_masked_multi_sequence_pass_equals_each_sequence_alone():
    shape, w, prefix, cache, g = _setup(seed=2)
    drafts = g.integers(0, shape.vocab, (3, 4))
    both = O.verify_forward(shape, w, cache.copy(), drafts, rounding="ideal")
    for i in range(3):
        alone = O.verify_forward(shape, w, cache.copy(), drafts[i:i + 1], rounding="ideal")
        np.testing.assert_allclose(both[i * 4:(i + 1) * 4], alone, rtol=1e-10, atol=1e-12)
    # and each equals the brute-force uncached pass over prefix + that sequence
    for i in range(3):
        full = O.full_forward_uncached(shape, w, prefix + drafts[i].tolist())
        np.testing.assert_allclose(both[i * 4:(i + 1) * 4], full[len(prefix):], rtol=1e-9, atol=1e-11)


def test_root_row_variant_equals_uncached_pass():
    shape, w, prefix, cache, g = _setup(seed=3)
    drafts = g.integers(0, shape.vocab, (2, 3))
    root = 7
    lg = O.verify_forward(shape, w, cache.copy(), drafts, root_token=root, rounding="ideal")
    assert lg.shape[0] == 1 + 6
    for i in range(2):
        full = O.full_forward_uncached(shape, w, prefix + [root] + drafts[i].tolist())
        np.testing.assert_allclose(lg[0], full[len(prefix)], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(lg[1 + i * 3:1 + (i + 1) * 3], full[len(prefix) + 1:], rtol=1e-9, atol=1e-11)


def test_commit_then_verify_equals_prefill_then_verify():
    shape, w, prefix, cache, g = _setup(seed=4)
    drafts = g.integers(0, shape.vocab, (3, 4))
    c = cache.copy()
    O.verify_forward(shape, w, c, drafts, rounding="ideal")
    res = O.VerifyResult(np.array([1, 3, 0]), np.array([5, 9, 2]), 1, 3, 9, c.prefix_len + 3)
    O.commit_kv(c, res, 4, has_root=False)
    assert c.prefix_len == len(prefix) + 3
    nxt = g.integers(0, shape.vocab, (2, 3))
    a = O.verify_forward(shape, w, c, nxt, root_token=9, rounding="ideal")
    fresh = O.prefill(shape, w, prefix + drafts[1, :3].tolist(), max_seq=40, rounding="ideal")
    b = O.verify_forward(shape, w, fresh, nxt, root_token=9, rounding="ideal")
    np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-11)


def test_contract_rounding_stays_close_to_ideal_and_differs():
    from paper_2503_00784_amd import inputs
    shape_in = inputs.ModelShape(2, 64, 4, 2, 16, 96, 101)
    shape = O.shape_from(shape_in)
    w = inputs.make_weights(shape_in, seed=1, threads=2)
    toks = list(range(3, 15))
    ideal = O.full_forward_uncached(shape, w, toks, rounding="ideal")
    contract = O.full_forward_uncached(shape, w, toks, rounding="contract")
    err = np.abs(ideal - contract).max()
    assert 0 < err < 2e-2 * max(1.0, np.abs(ideal).max())
    cache = O.prefill(shape, w, toks[:8], max_seq=16, rounding="contract")
    lg = O.verify_forward(shape, w, cache, np.array([toks[8:]]), rounding="contract")
    np.testing.assert_allclose(lg, contract[8:], rtol=1e-9, atol=1e-11)


def test_row_plan_slots_positions_and_visibility():
    plan = O.row_plan(10, 2, 3, has_root=True)
    assert plan[0] == (10, 10, [0])
    assert plan[1] == (11, 11, [0, 1])
    assert plan[3] == (13, 13, [0, 1, 2, 3])
    assert plan[4] == (11, 14, [0, 4])
    assert plan[6] == (13, 16, [0, 4, 5, 6])
    plan = O.row_plan(10, 2, 2, has_root=False)
    assert plan == [(10, 10, [0]), (11, 11, [0, 1]), (10, 12, [2]), (11, 13, [2, 3])]


# ------------------------------------------------------------------ fp16 as the storage type (the paper's precision)
def test_fp16_rounding_and_generator_match_torch():
    import torch
    from paper_2503_00784_amd import inputs
    assert O.round_to_fp16(np.array([1.0 + 2.0 ** -11]))[0] == 1.0                   # tie -> even mantissa
    assert O.round_to_fp16(np.array([1.0 + 3 * 2.0 ** -11]))[0] == 1.0 + 2.0 ** -9
    x = np.random.default_rng(5).normal(size=4096).astype(np.float32)
    t = torch.from_numpy(x).to(torch.float16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_to_fp16(x), t)
    w = inputs.make_weights(inputs.ModelShape(1, 64, 4, 2, 16, 96, 50), seed=2, threads=2, dtype="fp16")
    b = inputs.make_weights(inputs.ModelShape(1, 64, 4, 2, 16, 96, 50), seed=2, threads=2)
    assert w["wq"][0].dtype == np.float16 and b["wq"][0].dtype == np.uint16
    # the same draws on two grids: equal to within the coarser (bf16) rounding step
    np.testing.assert_allclose(w["wq"][0].astype(np.float64), O.bf16_bits_to_f64(b["wq"][0]), rtol=2.0 ** -8, atol=0)
    np.testing.assert_array_equal(O.bf16_bits_to_f64(w["wq"][0]), w["wq"][0].astype(np.float64))


def test_fp16_parameters_only_change_widening_and_the_cache_grid():
    """With float16 parameters the forward pass is the same arithmetic on the widened values (ideal mode equals the pass
    over the same values given as float64), and the contract rounds what the cache stores to the fp16 grid."""
    from paper_2503_00784_amd import inputs
    shape_in = inputs.ModelShape(2, 64, 4, 2, 16, 96, 101)
    shape = O.shape_from(shape_in)
    w16 = inputs.make_weights(shape_in, seed=1, threads=2, dtype="fp16")
    w64 = {k: ([a.astype(np.float64) for a in v] if isinstance(v, list) else v.astype(np.float64)) for k, v in w16.items()}
    toks = list(range(3, 15))
    np.testing.assert_array_equal(O.full_forward_uncached(shape, w16, toks, rounding="ideal"),
                                  O.full_forward_uncached(shape, w64, toks, rounding="ideal"))
    cache = O.prefill(shape, w16, toks[:8], max_seq=16, rounding="contract")
    kept = cache.k[:, :, :8]
    np.testing.assert_array_equal(kept, kept.astype(np.float16).astype(np.float64))   # on the fp16 grid
    assert np.abs(kept - O.round_to_bf16(kept)).max() > 0                              # and not on the bf16 grid
    ideal = O.full_forward_uncached(shape, w16, toks, rounding="ideal")
    contract = O.full_forward_uncached(shape, w16, toks, rounding="contract")
    err = np.abs(ideal - contract).max()
    assert 0 < err < 3e-3 * max(1.0, np.abs(ideal).max())                             # fp16 cache: 8x finer than bf16
