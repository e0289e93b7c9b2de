"""Dynamic multi-sequence drafting (Sec. 3.2), host side.

The draft model itself is outside this library: it enters as a callable that maps a token list to
the draft distribution of the next token.  This module turns it into the inputs of duo_verify:
how many sequences to draft, which first tokens seed them, and the [s][k] token / [s][k][V]
distribution arrays.

Rule of Sec. 3.2, in this module's words: with p(1, j) the j-th largest draft probability at the
first position and p(2, 1) the largest probability at the second position of the top-1 path,
theta = p(1, 1) * p(2, 1) estimates the chance that the two most likely tokens are both accepted.
Every first-position token whose probability exceeds theta seeds its own sequence (the top-1
token always does); the draft budget gamma is shared, each of the s sequences gets gamma // s
tokens (Alg. 1 writes the shape as [s, gamma / s]).

Readings where the paper is silent: ties at exactly theta do not seed a sequence; the number of
sequences is capped so that every sequence has at least one token; tokens after the seed are the
draft model's most likely continuation unless uniforms are supplied, in which case they are
drawn from its distribution by inverse CDF.

Fidelity.  The sequential first-token rule of Alg. 2 (test each sequence's first token against the
running target distribution, replace that by its normalised residual after a rejection) reproduces
the target distribution when every first token is a DRAW from the draft distribution handed to the
verifier.  Seeds picked by rank (the paper's Fig. 2: the most likely first tokens, one sequence
each) are not draws from the first-position distribution, and verifying them against it is then not
distribution-preserving: the emitted token over-represents the seeds.  `sample_seeds=True` keeps the
rule's count of sequences but draws the s first tokens independently from the first-position
distribution with caller-supplied uniforms (repeats are possible and harmless); that is the
setting in which the sequential rule is lossless.  tests/test_drafting.py shows both facts.
"""
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

DraftStep = Callable[[List[int]], np.ndarray]


def sequence_threshold(first_probs: np.ndarray, second_top_prob: float) -> float:
    """theta = p(1, 1) * p(2, 1)."""
    return float(np.max(first_probs)) * float(second_top_prob)


def seed_tokens(first_probs: np.ndarray, second_top_prob: float, gamma: int, max_sequences: int = 0) -> List[int]:
    """First tokens of the draft sequences, most likely first: every token with probability above
    theta, at least the top-1 token, at most gamma (and max_sequences if given)."""
    if gamma < 1:
        raise ValueError("gamma must be at least 1")
    p = np.asarray(first_probs, dtype=np.float64)
    theta = sequence_threshold(p, second_top_prob)
    order = np.argsort(-p, kind="stable")
    seeds = [int(order[0])]
    for t in order[1:]:
        if not p[t] > theta:
            break
        seeds.append(int(t))
    cap = gamma if not max_sequences else min(gamma, max_sequences)
    return seeds[:max(1, cap)]


def _next_token(probs: np.ndarray, u: Optional[float]) -> int:
    if u is None:
        return int(np.argmax(probs))
    c = np.cumsum(np.asarray(probs, dtype=np.float64))
    idx = int(np.searchsorted(c, float(u) * c[-1], side="right"))
    return min(idx, len(c) - 1)


def build_draft_sequences(draft_step: DraftStep, prefix: Sequence[int], gamma: int, max_sequences: int = 0,
                          uniforms: Optional[np.ndarray] = None, sample_seeds: bool = False) -> Dict[str, object]:
    """Draft s sequences of k = gamma // s tokens after `prefix`.

    Returns {"tokens": int32 [s][k], "probs": float32 [s][k][V], "theta": float, "first_probs": the
    first-position distribution}.  probs[i][j] is the draft distribution that token (i, j) was taken
    from: for j = 0 the first-position distribution (shared by all sequences), which is what the
    verifier's residual updates need.  uniforms, if given, is [s][k] in [0, 1): entries (i, j >= 1)
    draw the continuation tokens.  The seeds are chosen by rank (the threshold rule) unless
    `sample_seeds` is set: then the rule still fixes how many sequences there are, but first token i
    is drawn from the first-position distribution by inverse CDF with uniforms[i][0] (required), the
    setting in which the verifier's sequential rule preserves the target distribution.
    """
    prefix = list(int(t) for t in prefix)
    q1 = np.asarray(draft_step(prefix), dtype=np.float64)
    top1 = int(np.argmax(q1))
    q2_top = np.asarray(draft_step(prefix + [top1]), dtype=np.float64)
    seeds = seed_tokens(q1, float(np.max(q2_top)), gamma, max_sequences)
    s = len(seeds)
    if sample_seeds:
        if uniforms is None:
            raise ValueError("sample_seeds needs uniforms[i][0] for the first tokens")
        seeds = [_next_token(q1, float(uniforms[i, 0])) for i in range(s)]
    k = max(1, gamma // s)
    V = q1.shape[0]
    tokens = np.zeros((s, k), dtype=np.int32)
    probs = np.zeros((s, k, V), dtype=np.float32)
    for i, seed in enumerate(seeds):
        seq = [seed]
        probs[i, 0] = q1
        for j in range(1, k):
            q = q2_top if (j == 1 and seed == top1) else np.asarray(draft_step(prefix + seq), dtype=np.float64)
            probs[i, j] = q
            seq.append(_next_token(q, None if uniforms is None else float(uniforms[i, j])))
        tokens[i] = seq
    return {"tokens": tokens, "probs": probs, "theta": sequence_threshold(q1, float(np.max(q2_top))),
            "first_probs": q1.astype(np.float32)}
