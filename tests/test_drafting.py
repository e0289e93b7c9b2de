"""Dynamic multi-sequence drafting (Sec. 3.2): the threshold rule on hand-made distributions and a
bigram toy draft model (no GPU)."""
import numpy as np
import pytest
from scipy import stats

from oracle import duo_oracle as O
from paper_2503_00784_amd import drafting


def test_threshold_and_seeds_on_a_worked_example():
    # p(1, .) = 0.5, 0.3, 0.15, 0.05 and p(2, 1) = 0.4: theta = 0.2 -> tokens with p > 0.2 seed sequences
    q1 = np.array([0.05, 0.5, 0.15, 0.3])
    assert drafting.sequence_threshold(q1, 0.4) == pytest.approx(0.2)
    assert drafting.seed_tokens(q1, 0.4, gamma=24) == [1, 3]
    # a confident second position raises theta: only the top-1 path remains
    assert drafting.seed_tokens(q1, 0.9, gamma=24) == [1]
    # an uncertain second position lowers it: three sequences (0.05 is not above theta = 0.05)
    assert drafting.seed_tokens(q1, 0.1, gamma=24) == [1, 3, 2]
    # caps: budget and explicit limit
    assert drafting.seed_tokens(q1, 0.1, gamma=2) == [1, 3]
    assert drafting.seed_tokens(q1, 0.1, gamma=24, max_sequences=1) == [1]
    with pytest.raises(ValueError):
        drafting.seed_tokens(q1, 0.1, gamma=0)


def _bigram(V, seed):
    g = np.random.default_rng(seed)
    logits = g.normal(0, 2.0, (V, V))
    table = np.exp(logits - logits.max(axis=1, keepdims=True))
    table /= table.sum(axis=1, keepdims=True)
    return table, (lambda toks: table[toks[-1]])


def test_sequences_from_a_bigram_draft_model():
    V, gamma = 40, 12
    table, step = _bigram(V, 1)
    prefix = [3, 7]
    out = drafting.build_draft_sequences(step, prefix, gamma)
    toks, probs = out["tokens"], out["probs"]
    s, k = toks.shape
    q1 = table[7]
    theta = q1.max() * table[int(np.argmax(q1))].max()
    assert out["theta"] == pytest.approx(theta)
    assert s == min(gamma, int((q1 > theta).sum()))  # the top-1 token always exceeds theta = p(1,1) * p(2,1)
    assert k == gamma // s and s * k <= gamma
    assert len(set(toks[:, 0].tolist())) == s and toks[0, 0] == int(np.argmax(q1))
    for i in range(s):
        np.testing.assert_allclose(probs[i, 0], q1, rtol=1e-6)
        for j in range(1, k):
            np.testing.assert_allclose(probs[i, j], table[toks[i, j - 1]], rtol=1e-6)  # drawn from the right context
            assert toks[i, j] == int(np.argmax(table[toks[i, j - 1]]))                 # greedy continuation
    # every seed beyond the first has first-position probability above theta
    assert all(q1[t] > theta for t in toks[1:, 0])


def test_sampled_continuations_follow_the_uniforms():
    V, gamma = 25, 8
    table, step = _bigram(V, 2)
    u = np.full((8, 8), 0.999)
    out = drafting.build_draft_sequences(step, [5], gamma, max_sequences=2, uniforms=u)
    toks = out["tokens"]
    for i in range(toks.shape[0]):
        for j in range(1, toks.shape[1]):
            c = np.cumsum(table[toks[i, j - 1]])
            assert toks[i, j] == min(int(np.searchsorted(c, 0.999 * c[-1], side="right")), V - 1)
    u0 = np.zeros((8, 8))
    toks0 = drafting.build_draft_sequences(step, [5], gamma, max_sequences=2, uniforms=u0)["tokens"]
    # u = 0 picks the first token with positive probability, i.e. id 0 for a full-support model
    assert (toks0[:, 1:] == 0).all()


def _first_emitted_histogram(sample_seeds, N, seed):
    """Draft with the constructor, verify with the oracle's sequential multi-sequence rule (Alg. 2), count the first
    emitted token.  One fixed context: draft distribution q1 at the first position, target distribution p."""
    g = np.random.default_rng(seed)
    V, gamma = 8, 6
    q1 = np.array([0.30, 0.26, 0.20, 0.10, 0.06, 0.04, 0.03, 0.01])
    q_next = g.dirichlet(np.ones(V) * 0.3)                      # the draft model's distribution at later positions
    q_next = np.maximum(q_next, 1e-3) / np.maximum(q_next, 1e-3).sum()   # top probability of about 0.5: theta ~ 0.15, three sequences
    p = g.dirichlet(np.ones(V) * 2.0)
    step = lambda toks: q1 if len(toks) == 1 else q_next
    logits_p = np.log(p).astype(np.float32)
    p_seen = O.target_probs(logits_p, 1.0)                      # what the oracle sees after the fp32 round trip
    counts = np.zeros(V)
    shapes = set()
    for _ in range(N):
        u_draft = g.random((gamma, gamma))
        out = drafting.build_draft_sequences(step, [0], gamma, uniforms=u_draft, sample_seeds=sample_seeds)
        toks, probs = out["tokens"], out["probs"]
        s, k = toks.shape
        shapes.add((s, k))
        logits = np.tile(logits_p, (s * k, 1))                   # every later position is judged by the same p: only the first token matters here
        u = g.random((s, k + 1)).astype(np.float32)
        res = O.speculative_verify(logits, logits_p, toks, probs, u, prefix_len=1, select_mode=O.MODE_PAPER_SEQUENTIAL)
        counts[toks[res.selected, 0] if res.selected >= 0 else res.commit_token] += 1
    return counts, p_seen, q1, shapes


def test_rank_seeded_first_tokens_are_not_distribution_preserving():
    """Seeds chosen by rank (one sequence per likely first token, as in Fig. 2) and verified against the shared
    first-position distribution: the emitted token does NOT follow the target, it over-represents the seeds."""
    N = 20000
    counts, p_seen, q1, shapes = _first_emitted_histogram(False, N, 11)
    assert all(s >= 2 for s, _ in shapes)                         # several sequences were drafted
    assert stats.chisquare(counts, p_seen * N).pvalue < 1e-6


def test_sampled_seeds_preserve_the_target_distribution():
    """The same constructor with sample_seeds=True (first tokens drawn from the first-position distribution): the
    sequential rule of Alg. 2 is lossless, the emitted token follows the target."""
    N = 40000
    counts, p_seen, q1, shapes = _first_emitted_histogram(True, N, 12)
    assert all(s >= 2 for s, _ in shapes)
    assert stats.chisquare(counts, p_seen * N).pvalue > 1e-3
    assert stats.chisquare(counts, q1 * N).pvalue < 1e-6          # power: it is far from the draft distribution


def test_sample_seeds_needs_uniforms():
    with pytest.raises(ValueError):
        drafting.build_draft_sequences(lambda t: np.ones(4) / 4, [0], 4, sample_seeds=True)
