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


def compare_end_to_end(res_gpu, res_ora, n):
    """Accept lengths must agree wherever the oracle's decision margin exceeds ACCEPT_TIE."""
    compared = 0
    for i in range(n):
        if res_ora.accept_margins[i] > ACCEPT_TIE:
            assert res_gpu["accept_len"][i] == res_ora.accept_len[i], (i, res_gpu["accept_len"], res_ora.accept_len)
            compared += 1
    return compared
