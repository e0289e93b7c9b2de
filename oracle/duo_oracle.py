"""CPU oracle for the target-side verification step of DuoDecoding (arxiv 2503.00784).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the HIP library never does, and this file
imports nothing from the HIP package.  Everything is plain numpy in float64, written from
the definitions, one row / one head at a time, with no blocking or fusion.

What it computes
  * `verify_forward`: the target pass p <- M_p(x) of Alg. 1 (right column) for n draft
    sequences of k tokens that branch from a shared prefix held in a KV cache.  A row sees
    the prefix, the optional shared root token and the earlier tokens of its own sequence
    only ("independent" sequences, Sec. 3.2 / Fig. 2).  The decoder is Llama-shaped
    (RMSNorm, rotary embedding with half-split pairs, grouped-query attention, SwiGLU),
    the architecture of the paper's targets (Sec. 4.1 "Models").
  * `speculative_verify`: Alg. 2 recast for one fused call -- chain verification of a
    sequence (token by token, as plain speculative sampling verifies one: Sec. 3.3) and the
    sequential first-token test over s sequences with residual updates (Alg. 2, the
    "verify multi-sequence drafts" block), including the all-rejected case.
  * `duodec_verify_alg2`: Alg. 2 in the paper's own deferred form (unverified suffix first,
    then first tokens of the new sequences), used to show the fused form is built from
    the same pieces.

Rounding.  The paper runs the target in FP16 (Sec. 4.1); this build's contract is bf16 weights
and a bf16 KV cache with everything else carried wide.  `rounding="contract"` rounds exactly
where bf16 is a storage format: the rotated keys and the values written to the cache (the
weights arrive as bf16 already); every activation stays float64.  `rounding="ideal"` rounds
nowhere.  Logits are handed to sampling as float32, sampling is float64.

Pins (tests/test_oracle_*.py): HF `transformers` LlamaForCausalLM in float64 (the library
the paper's implementation builds on), brute-force uncached causal attention, k sequential
single-token decodes, each sequence alone, closed-form acceptance rates, chi-square tests of
the emitted-token distribution.  Unpinned conventions are listed in the design notes
(RMSNorm epsilon, gain initialisation, temperature of the paper's runs).
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

MODE_INDEPENDENT_LONGEST = 0
MODE_PAPER_SEQUENTIAL = 1


# ----------------------------------------------------------------------------- 16-bit storage types
# Parameters and cache entries arrive either as bf16 bit patterns (uint16 arrays: this build's default contract) or
# as numpy float16 arrays (IEEE fp16, the format of the paper's runs, Sec. 4.1); the array's dtype says which.
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of 16-bit storage to float64: bf16 bit patterns (uint16) or float16 values."""
    if bits.dtype == np.float16:
        return bits.astype(np.float64)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def round_to_fp16(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding to the IEEE fp16 grid, result kept as float64."""
    return np.asarray(x, dtype=np.float64).astype(np.float16).astype(np.float64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding to the bf16 grid (via float32), result kept as float64."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float64).astype(np.float32))
    u = f.view(np.uint32)
    r = (u + (((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    f = round_to_bf16(x).astype(np.float32)
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _identity(x: np.ndarray) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


# ----------------------------------------------------------------------------- pieces
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * gain, over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(vec: np.ndarray, pos: int, theta: float) -> np.ndarray:
    """Rotary embedding of one head vector (length D) at integer position `pos`.

    Pair (d, d + D/2) is rotated by the angle pos * theta^(-2d/D), d = 0 .. D/2-1.
    """
    D = vec.shape[-1]
    half = D // 2
    d = np.arange(half, dtype=np.float64)
    ang = float(pos) * theta ** (-2.0 * d / D)
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = vec[..., :half], vec[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def softmax(x: np.ndarray) -> np.ndarray:
    e = np.exp(x - np.max(x))
    return e / np.sum(e)


# ----------------------------------------------------------------------------- model
@dataclasses.dataclass
class OracleShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5


def shape_from(obj) -> OracleShape:
    return OracleShape(*(getattr(obj, f.name) for f in dataclasses.fields(OracleShape)))


class OracleCache:
    """KV cache as float64 values, [layer][kv_head][slot][head_dim]; slots >= prefix_len are scratch."""

    def __init__(self, shape: OracleShape, max_seq: int):
        L, H, D = shape.n_layers, shape.n_kv_heads, shape.head_dim
        self.k = np.zeros((L, H, max_seq, D))
        self.v = np.zeros((L, H, max_seq, D))
        self.prefix_len = 0
        self.root_logits: Optional[np.ndarray] = None  # float32 [V]
        self.max_seq = max_seq

    @classmethod
    def from_bits(cls, shape: OracleShape, k_bits: np.ndarray, v_bits: np.ndarray, prefix_len: int,
                  root_logits: Optional[np.ndarray]) -> "OracleCache":
        c = cls.__new__(cls)
        c.k = bf16_bits_to_f64(k_bits)
        c.v = bf16_bits_to_f64(v_bits)
        c.prefix_len = int(prefix_len)
        c.root_logits = None if root_logits is None else np.asarray(root_logits, dtype=np.float32).copy()
        c.max_seq = k_bits.shape[2]
        return c

    def copy(self) -> "OracleCache":
        c = OracleCache.__new__(OracleCache)
        c.k, c.v = self.k.copy(), self.v.copy()
        c.prefix_len, c.max_seq = self.prefix_len, self.max_seq
        c.root_logits = None if self.root_logits is None else self.root_logits.copy()
        return c


def _w(weights: Dict[str, object], name: str, layer: Optional[int] = None) -> np.ndarray:
    a = weights[name] if layer is None else weights[name][layer]
    return bf16_bits_to_f64(a) if a.dtype in (np.uint16, np.float16) else np.asarray(a, dtype=np.float64)


def _storage_rounding(weights: Dict[str, object], rounding: str):
    """The rounding applied where the 16-bit type is a storage format (the KV cache write): that of the parameters'
    own type under the contract, none in `ideal` mode."""
    if rounding != "contract":
        return _identity
    return round_to_fp16 if np.asarray(weights["embed"]).dtype == np.float16 else round_to_bf16


def embed_rows(weights: Dict[str, object], tokens: Sequence[int]) -> np.ndarray:
    """x_r = E[token_r] as float64 [len(tokens), d]."""
    e = weights["embed"][np.asarray(tokens, dtype=np.int64)]
    return bf16_bits_to_f64(e) if e.dtype in (np.uint16, np.float16) else np.asarray(e, dtype=np.float64)


def row_plan(prefix_len: int, n_seq: int, k_draft: int, has_root: bool
             ) -> List[Tuple[int, int, List[int]]]:
    """For every row of the pass: (position, cache slot, rows it may attend to besides the prefix).

    Row 0 is the shared root token when present (position P, slot P).  Draft token (i, j)
    sits at position P + R + j and slot P + R + i*k + j (R = 1 with a root, else 0) and
    sees the root and the tokens (i, j') with j' <= j of its own sequence.
    """
    R = 1 if has_root else 0
    plan: List[Tuple[int, int, List[int]]] = []
    if has_root:
        plan.append((prefix_len, prefix_len, [0]))
    for i in range(n_seq):
        for j in range(k_draft):
            vis = ([0] if has_root else []) + [R + i * k_draft + jj for jj in range(j + 1)]
            plan.append((prefix_len + R + j, prefix_len + R + i * k_draft + j, vis))
    return plan


def verify_forward(shape: OracleShape, weights: Dict[str, object], cache: OracleCache,
                   draft_tokens: np.ndarray, root_token: int = -1, rounding: str = "contract"
                   ) -> np.ndarray:
    """One target pass over the rows of `row_plan`; returns logits float64 [R + n*k, V].

    Writes the K/V of every row into its cache slot (scratch region beyond prefix_len).
    Row r's logits are the target's next-token scores after that row's token.
    """
    rnd = _storage_rounding(weights, rounding)
    draft_tokens = np.asarray(draft_tokens)
    n_seq, k_draft = draft_tokens.shape
    has_root = root_token >= 0
    P = cache.prefix_len
    plan = row_plan(P, n_seq, k_draft, has_root)
    tokens = ([int(root_token)] if has_root else []) + [int(t) for t in draft_tokens.reshape(-1)]
    M = len(plan)
    if M and max(s for _, s, _ in plan) >= cache.max_seq:
        raise ValueError("cache capacity exceeded")
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    group = Hq // Hkv
    x = embed_rows(weights, tokens)

    for l in range(shape.n_layers):
        h = rmsnorm(x, _w(weights, "g_attn", l), shape.rms_eps)
        q = h @ _w(weights, "wq", l).T
        kk = h @ _w(weights, "wk", l).T
        vv = h @ _w(weights, "wv", l).T
        q = q.reshape(M, Hq, D)
        kk = kk.reshape(M, Hkv, D)
        vv = vv.reshape(M, Hkv, D)
        for r, (pos, slot, _) in enumerate(plan):
            q[r] = rope(q[r], pos, shape.rope_theta)
            kk[r] = rope(kk[r], pos, shape.rope_theta)
        for r, (_, slot, _) in enumerate(plan):
            cache.k[l, :, slot, :] = rnd(kk[r])   # the cache stores bf16
            cache.v[l, :, slot, :] = rnd(vv[r])
        attn = np.zeros((M, Hq, D))
        for r, (_, _, vis_rows) in enumerate(plan):
            vis_slots = [plan[rr][1] for rr in vis_rows]
            for a in range(Hq):
                kvh = a // group
                k_pre, v_pre = cache.k[l, kvh, :P], cache.v[l, kvh, :P]
                k_own, v_own = cache.k[l, kvh, vis_slots], cache.v[l, kvh, vis_slots]
                s = np.concatenate([k_pre @ q[r, a], k_own @ q[r, a]]) / np.sqrt(D)
                w = softmax(s)
                attn[r, a] = w[:P] @ v_pre + w[P:] @ v_own
        x = x + attn.reshape(M, Hq * D) @ _w(weights, "wo", l).T
        h2 = rmsnorm(x, _w(weights, "g_ffn", l), shape.rms_eps)
        x = x + (silu(h2 @ _w(weights, "w_gate", l).T) * (h2 @ _w(weights, "w_up", l).T)) @ _w(weights, "w_down", l).T
    return rmsnorm(x, _w(weights, "g_final"), shape.rms_eps) @ _w(weights, "lm_head").T


def prefill(shape: OracleShape, weights: Dict[str, object], tokens: Sequence[int], max_seq: int,
            rounding: str = "contract") -> OracleCache:
    """Build a cache by scoring `tokens` as one causal sequence from an empty cache."""
    cache = OracleCache(shape, max_seq)
    logits = verify_forward(shape, weights, cache, np.asarray(tokens, dtype=np.int64).reshape(1, -1),
                            rounding=rounding)
    cache.prefix_len = len(tokens)
    cache.root_logits = logits[-1].astype(np.float32)
    return cache


def full_forward_uncached(shape: OracleShape, weights: Dict[str, object], tokens: Sequence[int],
                          rounding: str = "ideal") -> np.ndarray:
    """Textbook causal decoder over a whole sequence, no cache, T x T attention matrix.

    Independent of `verify_forward` on purpose (matrix form, explicit triangular mask): it is
    the brute-force pin for the cached, row-by-row pass.
    """
    rnd = _storage_rounding(weights, rounding)
    T = len(tokens)
    Hq, Hkv, D = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    x = embed_rows(weights, tokens)
    mask = np.tril(np.ones((T, T), dtype=bool))
    for l in range(shape.n_layers):
        h = rmsnorm(x, _w(weights, "g_attn", l), shape.rms_eps)
        q = (h @ _w(weights, "wq", l).T).reshape(T, Hq, D)
        k = (h @ _w(weights, "wk", l).T).reshape(T, Hkv, D)
        v = rnd((h @ _w(weights, "wv", l).T).reshape(T, Hkv, D))
        q = np.stack([rope(q[t], t, shape.rope_theta) for t in range(T)])
        k = rnd(np.stack([rope(k[t], t, shape.rope_theta) for t in range(T)]))
        out = np.zeros((T, Hq, D))
        for a in range(Hq):
            kvh = a // (Hq // Hkv)
            s = q[:, a, :] @ k[:, kvh, :].T / np.sqrt(D)
            s = np.where(mask, s, -np.inf)
            s = s - s.max(axis=1, keepdims=True)
            e = np.exp(s)
            out[:, a, :] = (e / e.sum(axis=1, keepdims=True)) @ v[:, kvh, :]
        x = x + out.reshape(T, Hq * D) @ _w(weights, "wo", l).T
        h2 = rmsnorm(x, _w(weights, "g_ffn", l), shape.rms_eps)
        x = x + (silu(h2 @ _w(weights, "w_gate", l).T) * (h2 @ _w(weights, "w_up", l).T)) @ _w(weights, "w_down", l).T
    return rmsnorm(x, _w(weights, "g_final"), shape.rms_eps) @ _w(weights, "lm_head").T


# ----------------------------------------------------------------------------- sampling
def nucleus(p: np.ndarray, top_p: float) -> Tuple[np.ndarray, float]:
    """Nucleus (top-p) restriction of one distribution: the most probable tokens, taken in order of
    decreasing probability (equal probabilities by ascending id), up to and including the one with
    which their mass reaches top_p; everything else set to zero and the rest renormalised.

    Returns (p', margin): margin is the distance of the running mass from the cut at the two positions
    that decide where the nucleus ends (a different summation order can only move the end when it is tiny).
    """
    p = np.asarray(p, dtype=np.float64)
    order = np.argsort(-p, kind="stable")
    c = np.cumsum(p[order])
    target = float(top_p) * c[-1]
    m = int(np.searchsorted(c, target, side="left"))  # first position whose running mass is >= target
    m = min(m, len(p) - 1)
    keep = order[:m + 1]
    out = np.zeros_like(p)
    out[keep] = p[keep] / p[keep].sum()
    before = c[m - 1] if m > 0 else 0.0
    return out, float(min(c[m] - target, target - before) / c[-1])


def target_probs(logits_f32: np.ndarray, temperature: float, top_p: float = 0.0) -> np.ndarray:
    """p = softmax(logits / T) in float64 from float32 logits.

    T = 0 is the limit T -> 0+: all mass on the largest logit, on the lowest id among equal ones
    (the greedy setting; Alg. 2 is then applied to this one-hot p without any other change).
    0 < top_p < 1 restricts every row to its nucleus (see `nucleus`); other values leave p as it is.
    """
    if 0.0 < float(top_p) < 1.0 and float(temperature) != 0.0:
        full = target_probs(logits_f32, temperature)
        if full.ndim == 1:
            return nucleus(full, top_p)[0]
        return np.stack([nucleus(r, top_p)[0] for r in full])
    l32 = np.asarray(logits_f32, dtype=np.float32)
    if float(temperature) == 0.0:
        p = np.zeros(l32.shape, dtype=np.float64)
        if l32.ndim == 1:
            p[int(np.argmax(l32))] = 1.0
        else:
            p[np.arange(l32.shape[0]), np.argmax(l32, axis=-1)] = 1.0
        return p
    z = l32.astype(np.float64) / float(temperature)
    return softmax(z)


def accept(u: float, q_t: float, p_t: float) -> bool:
    """Accept with probability min(1, p/q): u < p/q, evaluated without a division as u*q < p."""
    return float(u) * float(q_t) < float(p_t)


def residual_distribution(p: np.ndarray, q: np.ndarray) -> np.ndarray:
    """norm(max(0, p - q)); if the residual mass vanishes (p == q) fall back to p."""
    r = np.maximum(p - q, 0.0)
    R = r.sum()
    return r / R if R > 0.0 else p.copy()


def inverse_cdf(weights: np.ndarray, u: float) -> Tuple[int, float]:
    """Smallest token id v with sum_{w<=v} weights_w > u * sum(weights); ids ascending.

    Returns (token, relative margin to the nearer CDF edge).  If rounding leaves no such v,
    the largest id with a positive weight is taken.
    """
    c = np.cumsum(weights)
    total = c[-1]
    target = float(u) * total
    idx = int(np.searchsorted(c, target, side="right"))
    if idx >= len(weights):
        idx = int(np.max(np.nonzero(weights > 0)[0]))
        return idx, 0.0
    lo = c[idx - 1] if idx > 0 else 0.0
    margin = min(target - lo, c[idx] - target) / total
    return idx, float(margin)


@dataclasses.dataclass
class VerifyResult:
    accept_len: np.ndarray           # int32 [n]
    next_token: np.ndarray           # int32 [n]
    selected: int
    commit_len: int
    commit_token: int
    new_prefix_len: int
    # smallest relative margins of the decisions that shaped each sequence's outcome:
    # accept tests |u q - p| / p, and the inverse-CDF draw (distance to the nearer CDF edge / total)
    accept_margins: np.ndarray = None  # float64 [n]
    draw_margins: np.ndarray = None    # float64 [n]
    commit_margin: float = np.inf      # min over everything that decided the commit


def _chain(i: int, start: int, judge, q, tokens, u, k_draft: int) -> Tuple[int, float]:
    """Leading accepted positions j = start.. of sequence i; returns (first rejected j or k, margin)."""
    margin = np.inf
    j = start
    while j < k_draft:
        t = int(tokens[i, j])
        p_t, q_t = judge(i, j)[t], float(q[i, j, t])
        lhs = float(u[i, j]) * q_t
        margin = min(margin, abs(lhs - p_t) / max(p_t, 1e-300))
        if not accept(u[i, j], q_t, p_t):
            break
        j += 1
    return j, margin


def speculative_verify(logits_f32: np.ndarray, root_logits_f32: np.ndarray, draft_tokens: np.ndarray,
                       draft_probs: np.ndarray, uniforms: np.ndarray, prefix_len: int,
                       temperature: float = 1.0, select_mode: int = MODE_INDEPENDENT_LONGEST,
                       has_root: bool = False, top_p: float = 0.0) -> VerifyResult:
    """Speculative sampling over n sequences of k draft tokens (Alg. 2 recast; Sec. 3.3).

    logits_f32[(R +) i*k + j] scores the token after draft (i, j); the distribution judging
    draft (i, 0) is the root distribution (row 0 when `has_root`, else `root_logits_f32`),
    draft (i, j >= 1) is judged by row (i, j-1), the bonus token comes from row (i, k-1).
    uniforms[i][j] tests draft (i, j); uniforms[i][k] drives the correction / bonus sample.
    """
    tokens = np.asarray(draft_tokens)
    n, k = tokens.shape
    R = 1 if has_root else 0
    q = draft_probs
    u = np.asarray(uniforms, dtype=np.float32).astype(np.float64)
    p_root = target_probs(logits_f32[0] if has_root else root_logits_f32, temperature, top_p)
    cache_p: Dict[Tuple[int, int], np.ndarray] = {}

    def judge(i: int, j: int) -> np.ndarray:
        """Target distribution that judges draft (i, j); j == k is the bonus distribution."""
        if j == 0:
            return p_root
        if (i, j) not in cache_p:
            cache_p[(i, j)] = target_probs(logits_f32[R + i * k + j - 1], temperature, top_p)
        return cache_p[(i, j)]

    def finish(i: int, a: int) -> Tuple[int, float]:
        """Correction token after a rejection at position a, or bonus token when a == k."""
        pj = judge(i, a)
        if a < k:
            dist = residual_distribution(pj, np.asarray(q[i, a], dtype=np.float64))
        else:
            dist = pj
        return inverse_cdf(dist, u[i, k])

    accept_len = np.zeros(n, dtype=np.int32)
    next_token = np.full(n, -1, dtype=np.int32)
    margins = np.full(n, np.inf)
    draws = np.full(n, np.inf)

    if select_mode == MODE_INDEPENDENT_LONGEST:
        for i in range(n):
            a, m = _chain(i, 0, judge, q, tokens, u, k)
            tok, m2 = finish(i, a)
            accept_len[i], next_token[i], margins[i], draws[i] = a, tok, m, m2
        sel = int(np.argmax(accept_len))  # lowest index among the longest
        return VerifyResult(accept_len, next_token, sel, int(accept_len[sel]), int(next_token[sel]),
                            prefix_len + R + int(accept_len[sel]), margins, draws,
                            float(min(margins.min(), draws[sel])))

    if select_mode != MODE_PAPER_SEQUENTIAL:
        raise ValueError("unknown select_mode")
    # sequential test of the first token of each sequence against the running residual of p_root
    p_run = p_root
    commit_margin = np.inf
    sel = -1
    for i in range(n):
        t = int(tokens[i, 0])
        q0 = np.asarray(q[i, 0], dtype=np.float64)
        lhs = u[i, 0] * q0[t]
        m0 = abs(lhs - p_run[t]) / max(p_run[t], 1e-300)
        margins[i] = m0
        commit_margin = min(commit_margin, m0)
        if accept(u[i, 0], q0[t], p_run[t]):
            sel = i
            break
        p_run = residual_distribution(p_run, q0)
    if sel < 0:
        tok, m2 = inverse_cdf(p_run, u[n - 1, k])
        draws[:] = m2
        return VerifyResult(accept_len, next_token, -1, 0, tok, prefix_len + R, margins, draws,
                            float(min(commit_margin, m2)))
    a, m = _chain(sel, 1, judge, q, tokens, u, k)
    tok, m2 = finish(sel, a)
    accept_len[sel] = a
    next_token[sel] = tok
    accept_len[sel + 1:] = -1
    margins[sel] = min(margins[sel], m)
    draws[sel] = m2
    return VerifyResult(accept_len, next_token, sel, a, tok, prefix_len + R + a, margins, draws,
                        float(min(commit_margin, m, m2)))


def commit_kv(cache: OracleCache, res: VerifyResult, k_draft: int, has_root: bool) -> None:
    """Move the selected sequence's accepted K/V next to the prefix and advance prefix_len.

    The emitted token is not in the cache: the next pass scores it as the root token.
    """
    P, R = cache.prefix_len, (1 if has_root else 0)
    if res.selected >= 0:
        for j in range(res.commit_len):
            src = P + R + res.selected * k_draft + j
            dst = P + R + j
            cache.k[:, :, dst, :] = cache.k[:, :, src, :]
            cache.v[:, :, dst, :] = cache.v[:, :, src, :]
    cache.prefix_len = P + R + res.commit_len
    cache.root_logits = None


def oracle_verify(shape: OracleShape, weights: Dict[str, object], cache: OracleCache,
                  draft_tokens: np.ndarray, draft_probs: np.ndarray, uniforms: np.ndarray,
                  temperature: float = 1.0, select_mode: int = MODE_INDEPENDENT_LONGEST,
                  root_token: int = -1, rounding: str = "contract", top_p: float = 0.0
                  ) -> Tuple[VerifyResult, np.ndarray]:
    """The whole step: target pass, speculative sampling, KV commit.  Returns (result, fp32 logits)."""
    P = cache.prefix_len
    logits = verify_forward(shape, weights, cache, draft_tokens, root_token, rounding).astype(np.float32)
    res = speculative_verify(logits, cache.root_logits, draft_tokens, draft_probs, uniforms, P,
                             temperature, select_mode, has_root=root_token >= 0, top_p=top_p)
    k_draft = np.asarray(draft_tokens).shape[1]
    commit_kv(cache, res, k_draft, root_token >= 0)
    return res, logits


# ----------------------------------------------------------------------------- Alg. 2, deferred form
def duodec_verify_alg2(x: List[int], x_tilde: List[int], q_unverified: Sequence[np.ndarray],
                       p_unverified: Sequence[np.ndarray], p_n: np.ndarray,
                       xhat: Sequence[Sequence[int]], qhat0: Sequence[np.ndarray],
                       r_unverified: Sequence[float], r_seq: Sequence[float], r_final: float
                       ) -> Tuple[List[int], List[int]]:
    """Alg. 2 as the paper states it, for one iteration of the pipelined loop.

    x ends with the l = len(x_tilde) unverified tokens.  p_unverified[m] / q_unverified[m] are
    the target / draft distributions that judge x_tilde[m] (m = 0 is the earliest), p_n is the
    target distribution after the last token of x.  xhat[i] is new draft sequence i and
    qhat0[i] the draft distribution its first token was drawn from.  Returns (x, x_tilde).

    Reading of the listing: the earliest rejected unverified token is replaced by a sample
    from norm(max(0, p - q)) and everything after it is dropped; with none rejected the first
    token of each new sequence is tested in order against p_n, which is replaced by its
    residual after every rejection; an accepted sequence is appended whole and its tail
    becomes the new unverified suffix; if none is accepted a token is drawn from the final
    residual.
    """
    l = len(x_tilde)
    base = len(x) - l
    for m in range(l):
        t = x_tilde[m]
        if not accept(r_unverified[m], q_unverified[m][t], p_unverified[m][t]):
            tok, _ = inverse_cdf(residual_distribution(p_unverified[m], q_unverified[m]), r_final)
            return x[:base + m] + [tok], []
    p_run = p_n
    for i, seq in enumerate(xhat):
        t = seq[0]
        if accept(r_seq[i], qhat0[i][t], p_run[t]):
            return x + list(seq), list(seq[1:])
        p_run = residual_distribution(p_run, qhat0[i])
    tok, _ = inverse_cdf(p_run, r_final)
    return x + [tok], []
