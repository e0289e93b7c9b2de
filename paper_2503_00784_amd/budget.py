"""Draft budget from measured verify latencies (Sec. 3.1, hardware-aware draft budget).

The paper sets the number of draft tokens per round to the cost coefficient
c = T_target / T_draft: the draft model produces tokens for as long as one target pass takes,
so that neither side waits.  T_target is not quite flat in the number of verified tokens k, so
with a measured curve T_target(k) the balanced budget is the largest k for which drafting k
tokens still fits into the pass that verifies them: k * T_draft <= T_target(k).

Host-side arithmetic only (no GPU code): the curve comes from timing duo_verify at several k.
"""
from typing import Dict, Sequence, Tuple


def interpolate_latency(curve: Sequence[Tuple[int, float]], k: float) -> float:
    """Piecewise-linear T_target(k) through the measured (k, ms) points; flat outside the range."""
    pts = sorted(curve)
    if not pts:
        raise ValueError("empty latency curve")
    if k <= pts[0][0]:
        return pts[0][1]
    for (k0, t0), (k1, t1) in zip(pts, pts[1:]):
        if k <= k1:
            return t0 + (t1 - t0) * (k - k0) / (k1 - k0)
    return pts[-1][1]


def cost_coefficient(curve: Sequence[Tuple[int, float]], draft_step_ms: float) -> Dict[int, float]:
    """c(k) = T_target(k) / T_draft at every measured k."""
    if not draft_step_ms > 0:
        raise ValueError("draft_step_ms must be positive")
    return {int(k): t / draft_step_ms for k, t in sorted(curve)}


def draft_budget(curve: Sequence[Tuple[int, float]], draft_step_ms: float, k_max: int = 0) -> int:
    """Largest integer budget gamma >= 1 with gamma * T_draft <= T_target(gamma).

    k_max bounds the search (default: the largest measured k; beyond the measured range the
    curve is taken as flat, which is the paper's assumption for the whole range)."""
    if not draft_step_ms > 0:
        raise ValueError("draft_step_ms must be positive")
    pts = sorted(curve)
    hi = int(k_max) if k_max else int(pts[-1][0])
    gamma = 1
    for k in range(1, hi + 1):
        if k * draft_step_ms <= interpolate_latency(pts, k):
            gamma = k
    return gamma
