"""A verify step captured in a HIP graph (how bench.py launches it): every replay must reproduce the eager step bit for
bit, with the program's own eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2503_00784_amd import inputs
from tests.gpu_util import say, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2503_00784_amd import binding
    binding.load()
    return binding


@pytest.mark.parametrize("n,k,mode,root", [(1, 8, 0, -1), (4, 8, 0, 7), (3, 5, 1, -1), (8, 8, 0, -1)])
def test_graph_replays_match_the_eager_step(B, n, k, mode, root):
    import torch
    shape = inputs.MID
    P = 150
    say(f"graph replay n={n} k={k} mode={mode} root={root}")
    w = inputs.make_weights(shape, seed=8, threads=16)
    eng = B.VerifyEngine(shape, w, 256)
    kb, vb, rl = inputs.make_synthetic_cache(shape, P, 256, seed=8)
    eng.load_cache(kb, vb, P, rl)
    q, toks, u = inputs.make_draft(shape.vocab, n, k, seed=21, easy_rows=inputs.easy_rows_for(n, k))
    d_toks, d_q, d_u = to_dev(toks), to_dev(q), to_dev(u)
    R = 1 if root >= 0 else 0
    logits = torch.empty((R + n * k, shape.vocab), dtype=torch.float32, device="cuda")

    def step():
        eng.set_prefix_len(P)  # the previous step's commit advanced it
        eng.verify(d_toks, d_q, d_u, select_mode=mode, root_token=root, logits_out=logits)

    def snapshot():
        torch.cuda.synchronize()
        r = eng.results(n)
        kc, vc = eng.cache_to_host()
        return logits.cpu().numpy().copy(), r, kc[:, :, :P + R + n * k].copy(), vc[:, :, :P + R + n * k].copy()

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step()
        stream.synchronize()
        ref = snapshot()
        assert ref[1]["status"] == 0
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step()
        for rep in range(3):
            logits.fill_(float("nan"))        # eager work between the replays
            eng.load_cache(kb, vb, P, rl)     # the commit moved cache rows: restore the state the step started from
            stream.synchronize()
            graph.replay()
            got = snapshot()
            np.testing.assert_array_equal(got[0], ref[0])
            for key in ("status", "selected", "commit_len", "commit_token", "new_prefix_len", "device_prefix_len"):
                assert got[1][key] == ref[1][key], (rep, key)
            np.testing.assert_array_equal(got[1]["accept_len"], ref[1]["accept_len"])
            np.testing.assert_array_equal(got[1]["next_token"], ref[1]["next_token"])
            np.testing.assert_array_equal(got[2], ref[2])
            np.testing.assert_array_equal(got[3], ref[3])
