"""The entry point that allocates nothing (duo_spec_sample_noalloc, scratch in a static device array) against the
entry point it is a variant of (duo_spec_sample, scratch in the caller's workspace), through the C ABI: two calls
in a row on the same sampler object, the second with a smaller input, so that whatever the first call left in the
shared array is there when the second one runs.  Both are also held to the oracle, as every sampler test is."""
import numpy as np
import pytest

from oracle import duo_oracle as O
from paper_2503_00784_amd import inputs
from tests.gpu_util import say, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2503_00784_amd import binding
    binding.load()
    return binding


def _case(V, n, k, seed, has_root):
    g = np.random.default_rng(seed)
    R = 1 if has_root else 0
    logits = g.normal(0, 3.0, (R + n * k, V)).astype(np.float32)
    root = g.normal(0, 3.0, V).astype(np.float32)
    q, toks, u = inputs.make_draft(V, n, k, seed=seed, easy_rows=inputs.easy_rows_for(n, k))
    for i in range(n):  # drafts that often agree with the target, so that accepted lengths are not all zero
        for j in range(k):
            if g.random() < 0.6:
                jr = (logits[0] if has_root else root) if j == 0 else logits[R + i * k + j - 1]
                toks[i, j] = int(np.argmax(jr))
    return logits, root, q, toks, u


def _same(got, ref):
    np.testing.assert_array_equal(got["accept_len"], ref["accept_len"])
    np.testing.assert_array_equal(got["next_token"], ref["next_token"])
    for key in ("selected", "commit_len", "commit_token", "new_prefix_len", "status"):
        assert got[key] == ref[key], key


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("temperature", [1.0, 0.0])
def test_no_alloc_matches_workspace_entry_point_twice(B, mode, temperature):
    sampler = B.NoAllocSampler()
    # first a large call (128256-token vocabulary, 64 rows + root), then a smaller one in vocabulary, n and k
    for V, n, k, has_root, seed in [(128256, 4, 16, True, 1), (4099, 3, 5, False, 2)]:
        say(f"no-alloc sampler V={V} n={n} k={k} root={has_root} mode={mode} T={temperature}")
        logits, root, q, toks, u = _case(V, n, k, seed, has_root)
        dev = [to_dev(a) for a in (logits, root, toks, q, u)]
        ref = B.spec_sample(dev[0], dev[1], dev[2], dev[3], dev[4], temperature=temperature, select_mode=mode,
                            has_root=has_root, prefix_len=100)
        rc = sampler.run(dev[0], dev[1], dev[2], dev[3], dev[4], temperature=temperature, select_mode=mode,
                         has_root=has_root, prefix_len=100)
        assert rc == 0, B.status_string(rc)
        got = sampler.fetch(n)
        assert got["status"] == 0
        _same(got, ref)  # same kernels, same inputs, same order of additions: identical, ties included
        ora = O.speculative_verify(logits, root, toks, q, u, prefix_len=100, temperature=temperature, select_mode=mode,
                                   has_root=has_root)
        if ora.commit_margin > 1e-9 and (mode == 1 or min(ora.accept_margins.min(), ora.draw_margins.min()) > 1e-9):
            np.testing.assert_array_equal(got["accept_len"], ora.accept_len)
            np.testing.assert_array_equal(got["next_token"], ora.next_token)
            assert (got["selected"], got["commit_len"], got["commit_token"], got["new_prefix_len"]) == \
                   (ora.selected, ora.commit_len, ora.commit_token, ora.new_prefix_len)


def test_no_alloc_rejects_what_its_scratch_cannot_hold(B):
    sampler = B.NoAllocSampler()
    logits, root, q, toks, u = _case(50, 1, 2, 0, False)
    dev = [to_dev(a) for a in (logits, root, toks, q, u)]
    assert sampler.run(dev[0], dev[1], dev[2], dev[3], dev[4], top_p=0.9) == -9
    assert "scratch" in B.status_string(-9)
    assert sampler.run(dev[0], dev[1], dev[2], dev[3], dev[4]) == 0  # the refusal left nothing behind
    assert sampler.fetch(1)["status"] == 0
