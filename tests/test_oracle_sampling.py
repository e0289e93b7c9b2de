"""Pins for the oracle's speculative sampling: closed forms, special cases, distribution fidelity."""
import numpy as np
import pytest
from scipy import stats

from oracle import duo_oracle as O


def _dist(g, V, sharp=1.0):
    z = g.normal(size=V) * sharp
    e = np.exp(z - z.max())
    return e / e.sum()


def _logits(p):
    return np.log(p).astype(np.float32)


def _draw(g, dist):
    return int(min(np.searchsorted(np.cumsum(dist), g.random(), side="right"), len(dist) - 1))


def _f32_probs(p):
    """The distribution the oracle actually sees after the float32 logit round trip."""
    return O.target_probs(_logits(p), 1.0)


# ------------------------------------------------------------------ small deterministic pieces
def test_inverse_cdf_brute_force_and_edges():
    w = np.array([0.0, 0.2, 0.0, 0.5, 0.3, 0.0])
    for u in np.linspace(0, 0.999, 200):
        tok, margin = O.inverse_cdf(w, u)
        acc, want = 0.0, None
        for v in range(len(w)):
            acc += w[v]
            if acc > u * w.sum():
                want = v
                break
        assert tok == want and margin >= 0
    assert O.inverse_cdf(w, 0.0)[0] == 1          # never a zero-weight token
    assert O.inverse_cdf(w, 0.1999999)[0] == 1
    assert O.inverse_cdf(w, 0.2000001)[0] == 3
    assert O.inverse_cdf(w, 0.9999999)[0] == 4
    assert O.inverse_cdf(3.0 * w, 0.45)[0] == O.inverse_cdf(w, 0.45)[0]  # scale free
    assert O.inverse_cdf(np.array([0.5, 0.5, 0.0]), 1.0)[0] == 1  # rounding fallback: last positive


def test_residual_distribution_hand_values():
    p = np.array([0.5, 0.3, 0.2, 0.0])
    q = np.array([0.1, 0.6, 0.1, 0.2])
    np.testing.assert_allclose(O.residual_distribution(p, q), [0.8, 0.0, 0.2, 0.0], rtol=1e-15)
    np.testing.assert_array_equal(O.residual_distribution(p, p), p)  # vanishing residual -> p


def test_accept_rule_special_cases():
    assert O.accept(0.0, 0.5, 1e-30)            # u = 0 accepts anything with p > 0
    assert not O.accept(0.0, 0.5, 0.0)          # p = 0 never accepted
    assert O.accept(0.999, 0.0, 1e-30)          # q(t) = 0: accepted iff p > 0
    assert not O.accept(0.5, 0.0, 0.0)
    assert O.accept(0.49, 0.5, 0.25) and not O.accept(0.51, 0.5, 0.25) and not O.accept(0.5, 0.5, 0.25)
    assert O.accept(0.999999, 0.2, 0.3)         # p >= q: always accepted (u < 1)


def test_target_probs_temperature():
    lg = np.array([0.0, np.log(2.0), np.log(4.0)], dtype=np.float32)
    np.testing.assert_allclose(O.target_probs(lg, 1.0), np.array([1, 2, 4]) / 7.0, rtol=1e-6)
    np.testing.assert_allclose(O.target_probs(lg, 0.5), np.array([1, 4, 16]) / 21.0, rtol=1e-6)


def _single(p_rows, p_root, q, tokens, u, mode, has_root=False):
    logits = np.stack([_logits(r) for r in p_rows])
    return O.speculative_verify(logits, _logits(p_root), tokens, q, u, prefix_len=100,
                                temperature=1.0, select_mode=mode, has_root=has_root)


def test_p_equals_q_accepts_everything_and_bonus_follows_p():
    g = np.random.default_rng(0)
    V, k = 12, 4
    rows = [_dist(g, V) for _ in range(k)]
    root = _dist(g, V)
    judge = [root] + rows[:-1]
    q = np.stack([_f32_probs(j) for j in judge])[None]
    counts = np.zeros(V)
    for _ in range(3000):
        toks = np.array([[_draw(g, q[0, j]) for j in range(k)]])
        u = g.random((1, k + 1)).astype(np.float32)
        u[0, :k] = np.minimum(u[0, :k], np.float32(0.9999))  # q == p up to rounding: stay off the tie
        res = _single(rows, root, q, toks, u, O.MODE_INDEPENDENT_LONGEST)
        assert res.accept_len[0] == k and res.commit_len == k and res.new_prefix_len == 100 + k
        counts[res.commit_token] += 1
    pb = _f32_probs(rows[-1])
    assert stats.chisquare(counts, pb * counts.sum()).pvalue > 1e-3


def test_one_hot_draft():
    V, k = 6, 2
    root = np.array([0.1, 0.4, 0.2, 0.1, 0.1, 0.1])
    rows = [np.full(V, 1 / V)] * k
    q = np.zeros((1, k, V))
    q[0, :, 2] = 1.0
    toks = np.array([[2, 2]])
    # draft token 2 is accepted iff u < p(2) = 0.2
    res = _single(rows, root, q, toks, np.array([[0.19, 0.9, 0.5]], dtype=np.float32), 0)
    assert res.accept_len[0] == 1  # second: u=0.9 >= p(2)=1/6 -> rejected
    res = _single(rows, root, q, toks, np.array([[0.21, 0.0, 0.5]], dtype=np.float32), 0)
    assert res.accept_len[0] == 0
    # residual = p with entry 2 removed, renormalised: [.1,.4,0,.1,.1,.1]/.8 ; u=.5 -> cdf .125,.625 -> token 1
    assert res.next_token[0] == 1


def test_modes_agree_for_one_sequence():
    g = np.random.default_rng(7)
    V, k = 9, 5
    for trial in range(300):
        rows = [_dist(g, V) for _ in range(k)]
        root = _dist(g, V)
        q = np.stack([_dist(g, V, 0.5) for _ in range(k)])[None]
        toks = np.array([[_draw(g, q[0, j]) for j in range(k)]])
        u = g.random((1, k + 1)).astype(np.float32)
        a = _single(rows, root, q, toks, u, O.MODE_INDEPENDENT_LONGEST)
        b = _single(rows, root, q, toks, u, O.MODE_PAPER_SEQUENTIAL)
        assert (a.selected if a.commit_len else 0, a.commit_len, a.commit_token, a.new_prefix_len) == \
               (b.selected if b.commit_len else 0, b.commit_len, b.commit_token, b.new_prefix_len)


# ------------------------------------------------------------------ closed forms of the cited procedure
def test_acceptance_rate_is_sum_of_min_and_expected_length():
    g = np.random.default_rng(11)
    V, k, N = 10, 3, 20000
    p, q1 = _dist(g, V), _dist(g, V)
    pf = _f32_probs(p)
    alpha = np.minimum(pf, q1).sum()
    rows = [p] * k          # i.i.d. positions: every judging distribution is p, every draft q1
    q = np.tile(q1, (1, k, 1))
    lens = np.zeros(k + 1)
    for _ in range(N):
        toks = np.array([[_draw(g, q1) for _ in range(k)]])
        u = g.random((1, k + 1)).astype(np.float32)
        lens[_single(rows, p, q, toks, u, 0).accept_len[0]] += 1
    want = np.array([(1 - alpha) * alpha ** a for a in range(k)] + [alpha ** k]) * N
    assert stats.chisquare(lens, want).pvalue > 1e-3
    mean = (lens * np.arange(k + 1)).sum() / N
    closed = alpha * (1 - alpha ** k) / (1 - alpha)
    assert abs(mean - closed) < 4 * np.sqrt(k * k / N)


@pytest.mark.parametrize("mode", [O.MODE_INDEPENDENT_LONGEST, O.MODE_PAPER_SEQUENTIAL])
def test_first_emitted_token_follows_target_single_sequence(mode):
    """Emitted first token (accepted draft or correction) ~ p: the fidelity claim of the method."""
    g = np.random.default_rng(21 + mode)
    V, N = 12, 30000
    p, q1 = _dist(g, V, 1.5), _dist(g, V, 1.5)
    rows = [_dist(g, V)]
    counts = np.zeros(V)
    for _ in range(N):
        t = _draw(g, q1)
        u = g.random((1, 2)).astype(np.float32)
        res = _single(rows, p, q1[None, None], np.array([[t]]), u, mode)
        counts[t if res.commit_len >= 1 else res.commit_token] += 1
    assert stats.chisquare(counts, _f32_probs(p) * N).pvalue > 1e-3
    # power check: the same histogram is far from the draft distribution
    assert stats.chisquare(counts, q1 * N).pvalue < 1e-6


@pytest.mark.parametrize("n", [2, 3])
def test_first_emitted_token_follows_target_multi_sequence(n):
    """Sequential multi-sequence rule with i.i.d. first tokens drawn from their q: still ~ p."""
    g = np.random.default_rng(40 + n)
    V, N = 10, 30000
    p = _dist(g, V, 1.5)
    qs = [_dist(g, V, 1.5) for _ in range(n)]
    rows = [_dist(g, V)] * n
    counts = np.zeros(V)
    sel_hist = np.zeros(n + 1)
    for _ in range(N):
        toks = np.array([[_draw(g, qs[i])] for i in range(n)])
        u = g.random((n, 2)).astype(np.float32)
        res = _single(rows, p, np.stack(qs)[:, None, :], toks, u, O.MODE_PAPER_SEQUENTIAL)
        tok = toks[res.selected, 0] if res.selected >= 0 else res.commit_token
        counts[tok] += 1
        sel_hist[res.selected] += 1
    assert stats.chisquare(counts, _f32_probs(p) * N).pvalue > 1e-3
    assert sel_hist[:n].min() > 0 and sel_hist[n] > 0  # every branch of the rule was exercised


def test_keeping_p_instead_of_the_residual_breaks_fidelity():
    """Why the running distribution must be replaced by its residual after each rejection:
    a variant that keeps testing against the original p does not reproduce p."""
    g = np.random.default_rng(5)
    V, N, n = 6, 30000, 3
    p = _dist(g, V, 1.5)
    qs = [_dist(g, V, 1.5) for _ in range(n)]
    counts = np.zeros(V)
    for _ in range(N):
        p_run, out = p, None
        for i in range(n):
            t = _draw(g, qs[i])
            if O.accept(g.random(), qs[i][t], p[t]):      # wrong: p, not p_run
                out = t
                break
            p_run = O.residual_distribution(p_run, qs[i])
        if out is None:
            out = O.inverse_cdf(p_run, g.random())[0]
        counts[out] += 1
    assert stats.chisquare(counts, p * N).pvalue < 1e-6


def test_two_token_chain_joint_distribution_on_a_bigram_model():
    """Emitted pair (first, second) of a k = 2 chain follows p(x1) p(x2 | x1)."""
    g = np.random.default_rng(77)
    V, N = 5, 40000
    p1 = _dist(g, V)
    P2 = np.stack([_dist(g, V) for _ in range(V)])      # target bigram rows
    q1 = _dist(g, V)
    Q2 = np.stack([_dist(g, V) for _ in range(V)])      # draft bigram rows
    counts = np.zeros((V, V))
    for _ in range(N):
        t1 = _draw(g, q1)
        t2 = _draw(g, Q2[t1])
        u = g.random((1, 3)).astype(np.float32)
        rows = [P2[t1], _dist(g, V)]                    # row 0 scores after t1; row 1 is the bonus row
        q = np.stack([q1, Q2[t1]])[None]
        res = _single(rows, p1, q, np.array([[t1, t2]]), u, 0)
        if res.commit_len == 0:
            x1 = res.commit_token
            x2 = _draw(g, P2[x1])                       # next iteration would sample from the target
        elif res.commit_len == 1:
            x1, x2 = t1, res.commit_token
        else:
            x1, x2 = t1, t2
        counts[x1, x2] += 1
    want = (_f32_probs(p1)[:, None] * np.stack([_f32_probs(r) for r in P2])) * N
    assert stats.chisquare(counts.ravel(), want.ravel()).pvalue > 1e-3


def test_paper_mode_bookkeeping():
    V, k, n = 4, 2, 3
    root = np.array([0.25, 0.25, 0.25, 0.25])
    rows = [np.array([0.7, 0.1, 0.1, 0.1])] * (n * k)
    q = np.zeros((n, k, V))
    q[:, :, :] = [0.1, 0.2, 0.3, 0.4]
    toks = np.array([[3, 0], [2, 0], [1, 0]])
    # seq 0: token 3, p/q = .25/.4 = .625, u=.7 -> reject. residual = max(p-q,0) = [.15,.05,0,0]/.2 = [.75,.25,0,0]
    # seq 1: token 2 has residual mass 0 -> reject. residual = max([.75,.25,0,0]-q,0) = [.65,.05,0,0]/.7
    # seq 2: token 1: p_run = .05/.7 = .0714, q = .2, ratio .357; u=.3 -> accept
    u = np.array([[0.7, 0, 0], [0.0, 0, 0], [0.3, 0.1, 0.5]], dtype=np.float32)
    res = _single(rows, root, q, toks, u, O.MODE_PAPER_SEQUENTIAL)
    assert res.selected == 2
    # second token of seq 2: token 0, judged by row (2,0): p=.7, q=.1 -> accepted; bonus from row (2,1), u=.5 -> token 0
    assert res.commit_len == 2 and res.commit_token == 0 and res.new_prefix_len == 102
    assert res.accept_len.tolist() == [0, 0, 2] and res.next_token.tolist() == [-1, -1, 0]
    # all rejected: seq 2 with u = .4 -> reject; final residual = max([.65,.05,0,0]/.7 - q, 0) -> [.8286,0,0,0] -> token 0
    u[2, 0] = 0.4
    u[2, 2] = 0.99
    res = _single(rows, root, q, toks, u, O.MODE_PAPER_SEQUENTIAL)
    assert (res.selected, res.commit_len, res.commit_token, res.new_prefix_len) == (-1, 0, 0, 100)
    # first accepted stops the scan: later sequences are marked unexamined
    u[0, 0] = 0.6
    res = _single(rows, root, q, toks, u, O.MODE_PAPER_SEQUENTIAL)
    assert res.selected == 0 and res.accept_len.tolist()[1:] == [-1, -1]


def test_longest_mode_picks_lowest_index_among_longest():
    V, k, n = 4, 2, 3
    root = np.array([0.25, 0.25, 0.25, 0.25])
    rows = [np.array([0.25, 0.25, 0.25, 0.25])] * (n * k)
    q = np.full((n, k, V), 0.25)
    toks = np.zeros((n, k), dtype=np.int64)
    u = np.full((n, k + 1), 0.5, dtype=np.float32)   # p == q: all accepted -> lengths 2,2,2
    res = _single(rows, root, q, toks, u, 0)
    assert res.accept_len.tolist() == [2, 2, 2] and res.selected == 0
    q[0, 1, 0] = 0.75  # seq 0 second token: p/q = 1/3 < u -> rejected
    q[0, 1, 1:] = 0.25 / 3
    res = _single(rows, root, q, toks, u, 0)
    assert res.accept_len.tolist() == [1, 2, 2] and res.selected == 1 and res.new_prefix_len == 102


def test_root_row_judges_first_tokens():
    V, k = 4, 1
    root_cache = np.array([0.97, 0.01, 0.01, 0.01])
    root_row = np.array([0.01, 0.97, 0.01, 0.01])
    logits = np.stack([_logits(root_row), _logits(np.full(V, 0.25))])
    q = np.full((1, 1, V), 0.25)
    u = np.array([[0.5, 0.5]], dtype=np.float32)
    res = O.speculative_verify(logits, _logits(root_cache), np.array([[1]]), q, u, 10, has_root=True)
    assert res.accept_len[0] == 1 and res.new_prefix_len == 10 + 1 + 1
    res = O.speculative_verify(logits, _logits(root_cache), np.array([[0]]), q, u, 10, has_root=True)
    assert res.accept_len[0] == 0


# ------------------------------------------------------------------ Alg. 2 in the paper's deferred form
def test_deferred_form_pieces_match_the_fused_call():
    g = np.random.default_rng(9)
    V, n = 7, 3
    for trial in range(300):
        p_n = _dist(g, V)
        qs = [_dist(g, V) for _ in range(n)]
        seqs = [[_draw(g, qs[i]), int(g.integers(V))] for i in range(n)]
        r_seq = g.random(n).astype(np.float32)
        r_final = np.float32(g.random())
        pf = _f32_probs(p_n)
        x, xt = O.duodec_verify_alg2([1, 2, 3], [], [], [], pf, seqs, qs, [], r_seq, r_final)
        # fused call, paper mode, judging only position 0 (k = 1)
        u = np.zeros((n, 2), dtype=np.float32)
        u[:, 0] = r_seq
        u[:, 1] = r_final
        rows = [_dist(g, V)] * n
        res = _single(rows, p_n, np.stack(qs)[:, None, :], np.array([[s[0]] for s in seqs]), u, 1)
        if res.selected >= 0:
            assert x == [1, 2, 3] + seqs[res.selected] and xt == seqs[res.selected][1:]
        else:
            assert x == [1, 2, 3, res.commit_token] and xt == []


def test_deferred_form_unverified_suffix_is_textbook_chain():
    g = np.random.default_rng(10)
    V, l = 6, 3
    for trial in range(300):
        ps = [_f32_probs(_dist(g, V)) for _ in range(l)]
        qs = [_dist(g, V) for _ in range(l)]
        xt = [_draw(g, qs[m]) for m in range(l)]
        r = g.random(l).astype(np.float32)
        rf = np.float32(g.random())
        x, new_xt = O.duodec_verify_alg2([9] + xt, xt, qs, ps, _f32_probs(_dist(g, V)), [], [], r, [], rf)
        # fused call on the same chain: judging rows are ps[0] (root) and ps[1:], bonus row unused on rejection
        logits = np.stack([np.log(ps[m]).astype(np.float32) for m in range(1, l)] + [_logits(_dist(g, V))])
        u = np.concatenate([r, [rf]]).astype(np.float32)[None]
        res = O.speculative_verify(logits, np.log(ps[0]).astype(np.float32), np.array([xt]), np.stack(qs)[None], u, 1)
        if res.commit_len < l:
            assert x[:1 + res.commit_len] == [9] + xt[:res.commit_len]
            assert len(x) == 2 + res.commit_len and new_xt == []
            # log/exp round trip of float32 logits can move a CDF edge by ~1e-7: compare away from edges
            if res.commit_margin > 1e-5:
                assert x[-1] == res.commit_token
        else:
            assert x[:1 + l] == [9] + xt


# ------------------------------------------------------------------ the greedy limit (temperature 0)
def _greedy_case(g, V, n, k, match):
    """Random logits; sequence i copies the arg max of its judging rows for match[i] positions, then deviates."""
    logits = g.normal(size=(n * k, V)).astype(np.float32)
    root = g.normal(size=V).astype(np.float32)
    toks = np.zeros((n, k), dtype=np.int64)
    for i in range(n):
        for j in range(k):
            row = root if j == 0 else logits[i * k + j - 1]
            best = int(np.argmax(row))
            toks[i, j] = best if j < match[i] else (best + 1 + int(g.integers(V - 1))) % V
    q = np.stack([[_dist(g, V) for _ in range(k)] for _ in range(n)])
    return logits, root, toks, q


def test_greedy_target_probs_is_one_hot_lowest_id_on_ties():
    lg = np.array([0.5, 2.0, -1.0, 2.0], dtype=np.float32)
    assert O.target_probs(lg, 0.0).tolist() == [0.0, 1.0, 0.0, 0.0]
    two = O.target_probs(np.stack([lg, lg[::-1]]), 0.0)
    assert two.tolist() == [[0.0, 1.0, 0.0, 0.0], [1.0, 0.0, 0.0, 0.0]]


@pytest.mark.parametrize("mode", [O.MODE_INDEPENDENT_LONGEST, O.MODE_PAPER_SEQUENTIAL])
def test_greedy_is_prefix_match_with_the_arg_max_chain(mode):
    """Closed form of Alg. 2 at T = 0: the accepted length is the number of leading draft tokens equal to the target's
    arg max, the emitted token is the arg max after them, and no uniform can change that."""
    g = np.random.default_rng(11)
    V, k = 17, 5
    for n, match in ((1, [3]), (1, [5]), (1, [0]), (3, [0, 2, 4]), (3, [0, 0, 0]), (2, [5, 5])):
        logits, root, toks, q = _greedy_case(g, V, n, k, match)
        outs = []
        for useed in range(3):
            u = np.random.default_rng(useed).random((n, k + 1)).astype(np.float32)
            outs.append(O.speculative_verify(logits, root, toks, q, u, prefix_len=7, temperature=0.0, select_mode=mode))
        r = outs[0]
        for o in outs[1:]:
            assert (o.selected, o.commit_len, o.commit_token) == (r.selected, r.commit_len, r.commit_token)
        if mode == O.MODE_INDEPENDENT_LONGEST:
            assert r.accept_len.tolist() == match
            sel = int(np.argmax(match))                      # longest, lowest index among equals
        else:
            firsts = [i for i in range(n) if match[i] > 0]   # the first sequence whose first token is the arg max
            sel = firsts[0] if firsts else -1
        assert r.selected == sel
        length = match[sel] if sel >= 0 else 0
        assert r.commit_len == length and r.new_prefix_len == 7 + length
        row = root if length == 0 else logits[max(sel, 0) * k + length - 1]
        assert r.commit_token == int(np.argmax(row))


def test_greedy_equals_a_very_small_temperature():
    g = np.random.default_rng(12)
    V, n, k = 23, 2, 4
    for trial in range(5):
        logits, root, toks, q = _greedy_case(g, V, n, k, [int(g.integers(k + 1)) for _ in range(n)])
        u = g.random((n, k + 1)).astype(np.float32)
        for mode in (O.MODE_INDEPENDENT_LONGEST, O.MODE_PAPER_SEQUENTIAL):
            a = O.speculative_verify(logits, root, toks, q, u, prefix_len=0, temperature=0.0, select_mode=mode)
            b = O.speculative_verify(logits, root, toks, q, u, prefix_len=0, temperature=1e-4, select_mode=mode)
            assert (a.selected, a.commit_len, a.commit_token) == (b.selected, b.commit_len, b.commit_token)
            assert a.accept_len.tolist() == b.accept_len.tolist() and a.next_token.tolist() == b.next_token.tolist()


# ------------------------------------------------------------------ nucleus (top-p) restriction of the target
def _nucleus_by_hand(p, top_p):
    """The definition spelled out with a Python sort and a running sum."""
    order = sorted(range(len(p)), key=lambda v: (-p[v], v))
    total, run, keep = float(np.sum(p)), 0.0, []
    for v in order:
        keep.append(v)
        run += p[v]
        if run >= top_p * total:
            break
    out = np.zeros(len(p))
    out[keep] = p[keep] / np.sum(p[keep])
    return out


def test_nucleus_hand_values_and_ties_by_ascending_id():
    p = np.array([0.5, 0.2, 0.2, 0.1])
    out, _ = O.nucleus(p, 0.6)
    np.testing.assert_allclose(out, [5 / 7, 2 / 7, 0, 0], rtol=1e-15)     # of the two 0.2s the lower id is taken
    out, _ = O.nucleus(p, 0.45)
    assert out.tolist() == [1.0, 0.0, 0.0, 0.0]
    out, _ = O.nucleus(p, 0.95)
    np.testing.assert_allclose(out, p, rtol=1e-15)                          # everything is needed
    out, _ = O.nucleus(np.array([0.1, 0.4, 0.1, 0.4]), 0.5)
    np.testing.assert_allclose(out, [0, 0.5, 0, 0.5], rtol=1e-15)           # .4 (id 1) < .5, so id 3 joins


def test_nucleus_properties_and_brute_force():
    g = np.random.default_rng(31)
    for trial in range(200):
        V = int(g.integers(2, 40))
        p = _dist(g, V, sharp=float(g.uniform(0.3, 3.0)))
        if trial % 5 == 0:                       # some exact ties
            p[int(g.integers(V))] = p[int(g.integers(V))]
            p /= p.sum()
        top_p = float(g.uniform(0.05, 0.99))
        out, margin = O.nucleus(p, top_p)
        if margin < 1e-12:
            continue
        np.testing.assert_allclose(out, _nucleus_by_hand(p, top_p), rtol=1e-13, atol=0)
        kept = out > 0
        assert abs(out.sum() - 1.0) < 1e-12
        assert p[kept].sum() >= top_p * p.sum() - 1e-15                       # enough mass
        assert p[kept].sum() - p[kept].min() < top_p * p.sum() + 1e-15        # and no token too many
        if (~kept).any():
            assert p[kept].min() >= p[~kept].max()                            # the most probable ones
        np.testing.assert_allclose(out[kept] / out[kept].sum(), p[kept] / p[kept].sum(), rtol=1e-13)


def test_top_p_switched_off_and_its_greedy_limit():
    g = np.random.default_rng(32)
    V, n, k = 19, 2, 3
    logits = g.normal(size=(n * k, V)).astype(np.float32)
    root = g.normal(size=V).astype(np.float32)
    q = np.stack([[_dist(g, V) for _ in range(k)] for _ in range(n)])
    toks = g.integers(0, V, size=(n, k))
    toks[0, 0] = int(np.argmax(root))
    u = g.random((n, k + 1)).astype(np.float32)
    key = lambda r: (r.selected, r.commit_len, r.commit_token, r.accept_len.tolist(), r.next_token.tolist())
    for mode in (O.MODE_INDEPENDENT_LONGEST, O.MODE_PAPER_SEQUENTIAL):
        base = O.speculative_verify(logits, root, toks, q, u, 0, select_mode=mode)
        for off in (0.0, 1.0, 1.5, -0.3):
            assert key(O.speculative_verify(logits, root, toks, q, u, 0, select_mode=mode, top_p=off)) == key(base)
        greedy = O.speculative_verify(logits, root, toks, q, u, 0, temperature=0.0, select_mode=mode)
        tiny = O.speculative_verify(logits, root, toks, q, u, 0, select_mode=mode, top_p=1e-9)
        assert key(tiny) == key(greedy)         # a nucleus of one token is the arg max


def test_first_emitted_token_follows_the_nucleus_of_the_target():
    """With top-p the method must reproduce the RESTRICTED target distribution, and only that one."""
    g = np.random.default_rng(33)
    V, N, top_p = 12, 30000, 0.7
    p, q1 = _dist(g, V, 1.5), _dist(g, V, 1.5)
    rows = _logits(_dist(g, V))[None]
    want = O.nucleus(_f32_probs(p), top_p)[0]
    assert 2 <= (want > 0).sum() < V
    counts = np.zeros(V)
    for _ in range(N):
        t = _draw(g, q1)
        u = g.random((1, 2)).astype(np.float32)
        res = O.speculative_verify(rows, _logits(p), np.array([[t]]), q1[None, None], u, 0, top_p=top_p)
        counts[t if res.commit_len >= 1 else res.commit_token] += 1
    assert counts[want == 0].sum() == 0
    assert stats.chisquare(counts[want > 0], want[want > 0] * N).pvalue > 1e-3
    full = _f32_probs(p)
    assert stats.chisquare(counts[want > 0], full[want > 0] / full[want > 0].sum() * N).pvalue > 1e-3  # same shape inside
    assert abs(counts[int(np.argmax(full))] / N - full.max()) > 0.02           # but not the unrestricted probabilities
