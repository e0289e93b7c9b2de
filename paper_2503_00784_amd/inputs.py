"""Seeded synthetic inputs for the verify step (shared by the CPU oracle's tests and the HIP path).

This module only *draws* data: random bf16 weights, a synthetic prefix KV cache, draft
tokens, draft distributions and uniforms, in plain numpy arrays.  It holds none of the
method's arithmetic (no decoder layer, no attention, no acceptance rule) and imports
neither the oracle nor the HIP binding, so that both sides can be fed identical bytes
without sharing code.

Stand-in note: the paper evaluates on Spec-Bench and HumanEval with trained 7B targets and
a 68M draft model (Sec. 4.1).  Neither datasets nor weights are available here and the
latency of a verify step depends on shapes only, so these generators reproduce the shapes
(Llama-2-7B / Llama-3-8B decoder geometry, 32000 / 128256 vocabulary, draft budgets of
8-64 tokens around the paper's gamma = 24, 1-8 draft sequences) with random values.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Geometry of a Llama-shaped decoder (all matrices are [out, in], y = x W^T)."""

    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def weight_bytes(self) -> int:
        """bf16 bytes of every matrix the step streams once (embedding gather excluded)."""
        d, f = self.d_model, self.d_ff
        per_layer = (self.q_dim + 2 * self.kv_dim) * d + d * self.q_dim + 3 * d * f
        return 2 * (per_layer * self.n_layers + self.vocab * d)

    def kv_bytes_per_token(self) -> int:
        return 2 * 2 * self.n_layers * self.kv_dim


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    prefix_len: int
    n_seq: int
    k_draft: int

    def algorithmic_bytes(self) -> int:
        """Every weight once plus the shared-prefix KV once."""
        return self.shape.weight_bytes() + self.prefix_len * self.shape.kv_bytes_per_token()


TINY = ModelShape(2, 768, 12, 12, 64, 3072, 32000)
LLAMA2_7B = ModelShape(32, 4096, 32, 32, 128, 11008, 32000)
LLAMA3_8B = ModelShape(32, 4096, 32, 8, 128, 14336, 128256, rope_theta=500000.0)
# a mid-sized shape for parity tests that must span several tiles yet finish in seconds
MID = ModelShape(3, 512, 8, 2, 64, 1408, 4099)
# one 7B-wide layer (GQA, heads of 128): the launch shapes a prompt chunk of ~1000 rows takes at full width
WIDE1 = ModelShape(1, 4096, 32, 8, 128, 4096, 1000)
# one layer of 7B width exactly (32 heads of 128 without GQA, d_ff 11008): the launch shapes of the benchmark step
WIDE7 = ModelShape(1, 4096, 32, 32, 128, 11008, 1000)
# one layer of 13B width (d_model 5120, 40 heads, d_ff 13824): band counts and K ranges other than the 7B/8B ones
WIDE13 = ModelShape(1, 5120, 40, 40, 128, 13824, 1000)

WORKLOADS: Dict[str, Workload] = {
    "C0": Workload("C0-tiny-P128-n1-k8", TINY, 128, 1, 8),
    "C1": Workload("C1-llama2-7b-P512-n1-k8", LLAMA2_7B, 512, 1, 8),
    "C2": Workload("C2-llama2-7b-P2048-n4-k8", LLAMA2_7B, 2048, 4, 8),
    "C3": Workload("C3-llama2-7b-P4096-n8-k8", LLAMA2_7B, 4096, 8, 8),
    "C4": Workload("C4-llama3-8b-gqa-P8192-n4-k16", LLAMA3_8B, 8192, 4, 16),
}


# --------------------------------------------------------------------------- bf16 packing
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even packing of float32 values into bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def _rng(seed: int, *stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, *stream])))


def _normal_16(shape: Tuple[int, ...], std: float, mean: float, dtype: str, seed: int, *stream: int) -> np.ndarray:
    """Normal draws rounded to the 16-bit element type: bf16 bit patterns (uint16) or numpy float16."""
    g = _rng(seed, *stream)
    x = g.standard_normal(shape, dtype=np.float32)
    x *= np.float32(std)
    if mean != 0.0:
        x += np.float32(mean)
    return x.astype(np.float16) if dtype == "fp16" else f32_to_bf16_bits(x)


# tensor ids (second element of the seed sequence)
_T_EMBED, _T_LM, _T_GFINAL = 1, 2, 3
_T_LAYER = {"wq": 10, "wk": 11, "wv": 12, "wo": 13, "w_gate": 14, "w_up": 15, "w_down": 16,
            "g_attn": 17, "g_ffn": 18}
_T_PREFIX, _T_KV, _T_ROOT, _T_Q, _T_TOK, _T_UNI = 30, 31, 32, 33, 34, 35


def make_weights(shape: ModelShape, seed: int = 0, threads: int = 8, dtype: str = "bf16") -> Dict[str, object]:
    """Every parameter in the 16-bit element type: bf16 bit patterns (uint16 arrays) or, for dtype "fp16", numpy
    float16 arrays (the same draws, rounded to the other grid).

    Matrices, embedding and LM head ~ N(0, 0.02); RMSNorm gains ~ 1 + N(0, 0.02) (all-ones
    gains would hide a missing multiply).  Per-layer entries are lists of arrays.
    """
    d, f = shape.d_model, shape.d_ff
    dims = {"wq": (shape.q_dim, d), "wk": (shape.kv_dim, d), "wv": (shape.kv_dim, d),
            "wo": (d, shape.q_dim), "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
            "g_attn": (d,), "g_ffn": (d,)}
    jobs = []
    for name, dim in dims.items():
        for layer in range(shape.n_layers):
            gain = name.startswith("g_")
            jobs.append((name, layer, dim, 0.02, 1.0 if gain else 0.0, _T_LAYER[name]))
    jobs.append(("embed", None, (shape.vocab, d), 0.02, 0.0, _T_EMBED))
    jobs.append(("lm_head", None, (shape.vocab, d), 0.02, 0.0, _T_LM))
    jobs.append(("g_final", None, (d,), 0.02, 1.0, _T_GFINAL))

    def run(job):
        name, layer, dim, std, mean, tid = job
        return name, layer, _normal_16(dim, std, mean, dtype, seed, tid, 0 if layer is None else layer)

    out: Dict[str, object] = {name: [None] * shape.n_layers for name in dims}
    with ThreadPoolExecutor(max_workers=max(1, threads)) as pool:
        for name, layer, arr in pool.map(run, jobs):
            if layer is None:
                out[name] = arr
            else:
                out[name][layer] = arr
    return out


def make_prefix_ids(shape: ModelShape, prefix_len: int, seed: int = 0) -> np.ndarray:
    return _rng(seed, _T_PREFIX).integers(0, shape.vocab, size=prefix_len, dtype=np.int32)


def make_synthetic_cache(shape: ModelShape, prefix_len: int, max_seq: int, seed: int = 0, dtype: str = "bf16"
                         ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """A stand-in for a prefilled cache at sizes where a CPU prefill would take hours.

    K and V ~ N(0, 1.28^2) in bf16 for slots [0, prefix_len) (the statistics of a
    random-init projection of a unit-RMS input: sqrt(4096) * 0.02 = 1.28), zeros beyond;
    root logits ~ N(0, 1.28^2) fp32.  Layout [layer][kv_head][slot][head_dim].
    """
    L, H, D = shape.n_layers, shape.n_kv_heads, shape.head_dim
    host_type = np.float16 if dtype == "fp16" else np.uint16
    k = np.zeros((L, H, max_seq, D), dtype=host_type)
    v = np.zeros((L, H, max_seq, D), dtype=host_type)

    def fill(layer: int) -> None:
        k[layer, :, :prefix_len] = _normal_16((H, prefix_len, D), 1.28, 0.0, dtype, seed, _T_KV, layer, 0)
        v[layer, :, :prefix_len] = _normal_16((H, prefix_len, D), 1.28, 0.0, dtype, seed, _T_KV, layer, 1)

    with ThreadPoolExecutor(max_workers=8) as pool:
        list(pool.map(fill, range(L)))
    root = _rng(seed, _T_ROOT).standard_normal(shape.vocab, dtype=np.float32) * np.float32(1.28)
    return k, v, root


def make_draft(vocab: int, n_seq: int, k_draft: int, seed: int = 0, sharpness: float = 2.0,
               easy_rows: Optional[List[Tuple[int, int]]] = None
               ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Draft distributions q[n][k][V] (fp32), draft tokens[n][k] (int32), uniforms[n][k+1] (fp32).

    q_ij = exp(z) / sum(exp(z)) with z = sharpness * N(0,1); tokens are drawn from q_ij by
    inverse CDF.  For (i, j) in `easy_rows` the token is drawn uniformly over the vocabulary
    instead: such a token has a small draft probability, so it is accepted far more often
    than a q-sample, which makes acceptance lengths vary across sequences the way the
    argmax-copying sequences of the benchmark configurations do.
    """
    g = _rng(seed, _T_Q)
    z = g.standard_normal((n_seq, k_draft, vocab), dtype=np.float32) * np.float32(sharpness)
    z -= z.max(axis=-1, keepdims=True)
    e = np.exp(z.astype(np.float64))
    q = (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)
    gt = _rng(seed, _T_TOK)
    r = gt.random((n_seq, k_draft))
    uni_tok = gt.integers(0, vocab, size=(n_seq, k_draft))
    tokens = np.empty((n_seq, k_draft), dtype=np.int32)
    easy = set(easy_rows or [])
    for i in range(n_seq):
        for j in range(k_draft):
            if (i, j) in easy:
                tokens[i, j] = uni_tok[i, j]
            else:
                c = np.cumsum(q[i, j].astype(np.float64))
                tokens[i, j] = min(int(np.searchsorted(c, r[i, j] * c[-1], side="right")), vocab - 1)
    u = _rng(seed, _T_UNI).random((n_seq, k_draft + 1), dtype=np.float32)
    return q, tokens, u


def easy_rows_for(n_seq: int, k_draft: int) -> List[Tuple[int, int]]:
    """Even-numbered sequences get 'easy' tokens in their first four positions (n > 1 only)."""
    if n_seq == 1:
        return []
    return [(i, j) for i in range(0, n_seq, 2) for j in range(min(4, k_draft))]
