"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np

from oracle import duo_oracle as O
from paper_2503_00784_amd import binding as B
from paper_2503_00784_amd import inputs

LOGIT_ATOL, LOGIT_RTOL = 2e-2, 1e-2   # bf16 storage, wide accumulation: |g - o| <= atol + rtol * |o|
ACCEPT_TIE = 3e-2                      # an accept test closer than this (relative) can flip under LOGIT_ATOL


def say(*a):
    print(*a, flush=True)


def logits_close(gpu, ora):
    err = np.abs(gpu.astype(np.float64) - ora.astype(np.float64))
    bound = LOGIT_ATOL + LOGIT_RTOL * np.abs(ora)
    return bool((err <= bound).all()), float(err.max()), float((err / bound).max())


def to_dev(a, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def reachable_tokens(weights, u, delta):
    """Token ids whose CDF interval meets [u*total - delta*total, u*total + delta*total]."""
    c = np.cumsum(weights)
    total = c[-1]
    lo = np.searchsorted(c, (u - delta) * total, side="right")
    hi = np.searchsorted(c, (u + delta) * total, side="right")
    return int(max(lo, 0)), int(min(hi, len(weights) - 1))


def same_as_sampler_on(res_gpu, logits, root_logits, toks, q, u, prefix_len, temperature, mode, has_root, top_p=0.0):
    """The step's decisions against the oracle's sampler run on the logits the GPU itself returned: everything it
    emits (accepted lengths, correction / bonus tokens, the commit) must be identical, bit for bit, unless one of
    the oracle's own margins is within rounding of a tie (1e-9).  Returns whether the comparison was made."""
    ref = O.speculative_verify(logits, root_logits, toks, q, u, prefix_len=prefix_len, temperature=temperature,
                               select_mode=mode, has_root=has_root, top_p=top_p)
    if ref.commit_margin <= 1e-9 or (mode == 0 and min(ref.accept_margins.min(), ref.draw_margins.min()) <= 1e-9):
        return False
    np.testing.assert_array_equal(res_gpu["accept_len"], ref.accept_len)
    np.testing.assert_array_equal(res_gpu["next_token"], ref.next_token)
    assert (res_gpu["selected"], res_gpu["commit_len"], res_gpu["commit_token"], res_gpu["new_prefix_len"]) == \
           (ref.selected, ref.commit_len, ref.commit_token, ref.new_prefix_len)
    return True


def _draw_distribution(ora_logits, ora_root, q, i, a, k, R, temperature):
    """The distribution the correction (a < k) or bonus (a == k) token of sequence i is drawn from, on the oracle's logits."""
    row = (ora_logits[0] if R else ora_root) if a == 0 else ora_logits[R + i * k + a - 1]
    p = O.target_probs(row, temperature)
    return O.residual_distribution(p, np.asarray(q[i, a], dtype=np.float64)) if a < k else p


def compare_end_to_end(res_gpu, res_ora, n, mode=0, ora_logits=None, ora_root=None, q=None, u=None, k=None, R=0,
                       temperature=1.0):
    """The step's decisions against the oracle's step on its OWN logits, wherever the oracle's margins say that a
    logit difference within tolerance cannot move the decision (relative margin above ACCEPT_TIE): accepted lengths,
    the selected sequence, the commit, and emitted tokens whose inverse-CDF draw is that far from a CDF edge.  An
    emitted token whose draw is closer to an edge is checked for validity instead: it must lie in the id range the
    draw can reach when the CDF moves by ACCEPT_TIE.  Returns the number of sequences whose accepted length was
    compared (longest mode) or of first-token decisions compared (paper mode)."""
    compared = 0
    acc_g, acc_o = res_gpu["accept_len"], res_ora.accept_len

    def token_check(i, a, tok_gpu, tok_ora, margin):
        if margin > ACCEPT_TIE:
            assert tok_gpu == tok_ora, (i, tok_gpu, tok_ora)
        elif ora_logits is not None:
            lo, hi = reachable_tokens(_draw_distribution(ora_logits, ora_root, q, i, a, k, R, temperature), float(u[i, k]), ACCEPT_TIE)
            assert lo <= tok_gpu <= hi, (i, tok_gpu, lo, hi)

    if mode == 0:
        for i in range(n):
            if res_ora.accept_margins[i] > ACCEPT_TIE:
                assert acc_g[i] == acc_o[i], (i, acc_g, acc_o)
                compared += 1
                token_check(i, int(acc_o[i]), int(res_gpu["next_token"][i]), int(res_ora.next_token[i]), res_ora.draw_margins[i])
        if res_ora.accept_margins.min() > ACCEPT_TIE:
            assert (res_gpu["selected"], res_gpu["commit_len"]) == (res_ora.selected, res_ora.commit_len)
            if res_ora.draw_margins[res_ora.selected] > ACCEPT_TIE:
                assert res_gpu["commit_token"] == res_ora.commit_token
        return compared
    # paper mode: the first tokens are judged in index order; what follows a declared tie is not compared
    for i in range(n):
        if res_ora.accept_margins[i] <= ACCEPT_TIE:
            return compared
        compared += 1
        if res_ora.selected == i:  # margins[i] also covers the chain of the selected sequence
            assert res_gpu["selected"] == i and acc_g[i] == acc_o[i], (i, res_gpu["selected"], acc_g, acc_o)
            assert res_gpu["commit_len"] == res_ora.commit_len
            token_check(i, int(acc_o[i]), int(res_gpu["commit_token"]), int(res_ora.commit_token), res_ora.draw_margins[i])
            return compared
        assert res_gpu["selected"] != i and acc_g[i] == 0, (i, res_gpu["selected"], acc_g)
    assert res_gpu["selected"] == -1 and res_gpu["commit_len"] == 0  # every first token rejected, none near a tie
    if res_ora.draw_margins.min() > ACCEPT_TIE:
        assert res_gpu["commit_token"] == res_ora.commit_token
    return compared
