"""ctypes binding of libduo_verify.so: argument marshalling only.

Every step of the verify path runs in the HIP kernels behind the C ABI declared in
include/duo_verify.h; this module turns torch device tensors into raw pointers and back.
There is no CPU fallback: if the shared library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libduo_verify.so")            # bf16 weights and KV cache
LIB_PATH_FP16 = os.path.join(_HERE, "libduo_verify_fp16.so")  # the same sources built for IEEE fp16
LIB_PATHS = {"bf16": LIB_PATH, "fp16": LIB_PATH_FP16}

DUO_MAX_ROWS = 80
DUO_MAX_PREFILL_ROWS = 1024
SELECT_INDEPENDENT_LONGEST = 0
SELECT_PAPER_SEQUENTIAL = 1
STATUS_TOKEN_CLAMPED = 1
STATUS_PREFIX_MISMATCH = 2

EXPORTS = ["duo_workspace_bytes", "duo_verify", "duo_prefill_chunk", "duo_sample_workspace_bytes",
           "duo_spec_sample", "duo_spec_sample_noalloc", "duo_verify_deferred", "duo_deferred_sample", "duo_skinny_gemm",
           "duo_block_gemm", "duo_stream_read_probe", "duo_k_cache_offset",
           "duo_v_cache_offset", "duo_status_string", "duo_last_hip_error", "duo_profile_enable",
           "duo_profile_read", "duo_profile_dropped", "duo_profile_kernel_name", "duo_packed_elems", "duo_pack_matrix", "duo_pack_qkv", "duo_pack_gate_up",
           "duo_pack_activations"]
NOALLOC_MAX_VOCAB = 131072
PROF_CLASSES = ["setup", "qkv_rope", "attn", "attn_combine", "o_proj", "residual_reduce", "gate_up_swiglu", "down_proj", "lm_head",
                "sample", "commit", "qkv_finish"]

_u16p = C.POINTER(C.c_uint16)
_u16pp = C.POINTER(_u16p)


class ModelConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ff",
                                         "vocab", "max_seq")] + [("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p)] + [(n, C.POINTER(C.c_void_p)) for n in
                                          ("wqkv", "wo", "w_gate_up", "w_down", "g_attn", "g_ffn")] + \
               [("g_final", C.c_void_p), ("lm_head", C.c_void_p)]


class KVCache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("prefix_len", C.c_void_p), ("root_logits", C.c_void_p)]


class Call(C.Structure):
    _fields_ = [("n", C.c_int32), ("k", C.c_int32), ("temperature", C.c_float), ("select_mode", C.c_int32),
                ("root_token", C.c_int32), ("host_prefix_len", C.c_int32), ("top_p", C.c_float)]


class Result(C.Structure):
    _fields_ = [("accept_len", C.c_void_p), ("next_token", C.c_void_p), ("commit", C.c_void_p),
                ("status", C.c_void_p), ("logits_out", C.c_void_p)]


class DuoError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        self.code = code
        super().__init__(f"{where}: {detail} (code {code})")


_libs: Dict[str, C.CDLL] = {}


def dtype_of(host_array) -> str:
    """Element type of a host array of 16-bit parameters: numpy float16 arrays are fp16, uint16 arrays bf16 bit patterns."""
    return "fp16" if np.asarray(host_array).dtype == np.float16 else "bf16"


def load(dtype: str = "bf16") -> C.CDLL:
    """Load the shared library of one element type (once).  Raises if it has not been built."""
    if dtype in _libs:
        return _libs[dtype]
    path = LIB_PATHS[dtype]
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2503_00784_amd.build` "
                           "(there is no CPU fallback)")
    # The device memory and the streams handed to the library are torch's, so the library has to bind to the HIP
    # runtime that torch brought into the process; loading it first would bring in a second runtime (the system's),
    # which then finds no device.
    import torch  # noqa: F401
    lib = C.CDLL(path)
    lib.duo_workspace_bytes.argtypes = [C.POINTER(ModelConfig), C.c_int, C.POINTER(C.c_size_t)]
    lib.duo_verify.argtypes = [C.POINTER(ModelConfig), C.POINTER(Weights), C.POINTER(KVCache), C.c_void_p, C.c_void_p,
                               C.c_void_p, C.POINTER(Call), C.POINTER(Result), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.duo_prefill_chunk.argtypes = [C.POINTER(ModelConfig), C.POINTER(Weights), C.POINTER(KVCache), C.c_void_p, C.c_int,
                                      C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.duo_sample_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    lib.duo_spec_sample.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Call),
                                    C.POINTER(Result), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.duo_spec_sample_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Call),
                                            C.POINTER(Result), C.c_void_p]
    lib.duo_spec_sample_noalloc.restype = C.c_int
    lib.duo_profile_dropped.argtypes = []
    lib.duo_profile_dropped.restype = C.c_int
    lib.duo_profile_kernel_name.argtypes = [C.c_int]
    lib.duo_profile_kernel_name.restype = C.c_char_p
    lib.duo_verify_deferred.argtypes = [C.POINTER(ModelConfig), C.POINTER(Weights), C.POINTER(KVCache), C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                        C.POINTER(Call), C.POINTER(Result), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.duo_deferred_sample.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_int, C.POINTER(Call), C.POINTER(Result), C.c_void_p,
                                        C.c_size_t, C.c_void_p]
    lib.duo_skinny_gemm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
    lib.duo_block_gemm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
    lib.duo_stream_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    lib.duo_stream_read_probe.restype = C.c_int
    lib.duo_packed_elems.argtypes = [C.c_int, C.c_int]
    lib.duo_packed_elems.restype = C.c_size_t
    for name in ("duo_k_cache_offset", "duo_v_cache_offset"):
        getattr(lib, name).argtypes = [C.c_int, C.c_int, C.c_int]
        getattr(lib, name).restype = C.c_size_t
    lib.duo_pack_matrix.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    lib.duo_pack_qkv.argtypes = [C.POINTER(ModelConfig), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.duo_pack_gate_up.argtypes = [C.POINTER(ModelConfig), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.duo_pack_activations.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    for name in ("duo_workspace_bytes", "duo_verify", "duo_prefill_chunk", "duo_sample_workspace_bytes",
                 "duo_spec_sample", "duo_verify_deferred", "duo_deferred_sample", "duo_skinny_gemm", "duo_block_gemm", "duo_pack_matrix",
                 "duo_pack_qkv", "duo_pack_gate_up", "duo_pack_activations"):
        getattr(lib, name).restype = C.c_int
    lib.duo_profile_enable.argtypes = [C.c_int]
    lib.duo_profile_enable.restype = C.c_int
    lib.duo_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    lib.duo_profile_read.restype = C.c_int
    lib.duo_status_string.argtypes = [C.c_int]
    lib.duo_status_string.restype = C.c_char_p
    lib.duo_last_hip_error.argtypes = []
    lib.duo_last_hip_error.restype = C.c_char_p
    _libs[dtype] = lib
    return lib


def status_string(code: int) -> str:
    return load().duo_status_string(code).decode()


def _check(code: int, where: str) -> None:
    if code != 0:
        lib = load()
        detail = lib.duo_status_string(code).decode()
        if code == -7:
            detail += ": " + lib.duo_last_hip_error().decode()
        raise DuoError(code, where, detail)


def profile_enable(on: bool, dtype: str = "bf16") -> None:
    _check(load(dtype).duo_profile_enable(1 if on else 0), "duo_profile_enable")


def profile_dropped(dtype: str = "bf16") -> int:
    """Launches since the last read that went untimed because the event pool was empty (ask before profile_read)."""
    return int(load(dtype).duo_profile_dropped())


def profile_kernel_names(dtype: str = "bf16") -> Dict[str, str]:
    """{class: name of the kernel last launched under it while profiling} for the classes whose kernels are named."""
    lib = load(dtype)
    names = {c: lib.duo_profile_kernel_name(i).decode() for i, c in enumerate(PROF_CLASSES)}
    return {c: n for c, n in names.items() if n}


def profile_read(dtype: str = "bf16") -> Dict[str, Dict[str, float]]:
    """{class: {"ms": total milliseconds, "launches": count}} since the last read."""
    n = len(PROF_CLASSES)
    ms = (C.c_double * n)()
    cnt = (C.c_int32 * n)()
    _check(load(dtype).duo_profile_read(ms, cnt), "duo_profile_read")
    return {PROF_CLASSES[i]: {"ms": ms[i], "launches": cnt[i]} for i in range(n)}


def make_config(shape, max_seq: int) -> ModelConfig:
    return ModelConfig(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ff,
                       shape.vocab, max_seq, shape.rope_theta, shape.rms_eps)


def workspace_bytes(cfg: ModelConfig, max_rows: int) -> int:
    out = C.c_size_t(0)
    _check(load().duo_workspace_bytes(C.byref(cfg), max_rows, C.byref(out)), "duo_workspace_bytes")
    return out.value


# KV-cache layouts (the formulas of include/duo_verify.h as tensor reshapes; argument marshalling only).
# Row layout [..., slot, D] <-> tiled plane [..., max_seq * D].
def k_rows_to_tiles(k):
    """slot = (B, q, t, r) with w = 8q + 4t + r, channel = (ks, g, j)  ->  (B, t, ks, g, q, r, j)."""
    *lead, S, D = k.shape
    x = k.reshape(*lead, S // 32, 4, 2, 4, D // 32, 4, 8)
    n = len(lead)
    return x.permute(*range(n), n, n + 2, n + 4, n + 5, n + 1, n + 3, n + 6).contiguous().reshape(*lead, S * D)


def k_tiles_to_rows(kt, D):
    *lead, SD = kt.shape
    S = SD // D
    x = kt.reshape(*lead, S // 32, 2, D // 32, 4, 4, 4, 8)  # (B, t, ks, g, q, r, j)
    n = len(lead)
    return x.permute(*range(n), n, n + 4, n + 1, n + 5, n + 2, n + 3, n + 6).contiguous().reshape(*lead, S, D)


def v_rows_to_tiles(v):
    """slot = (B, g, j), channel = (dt, c)  ->  (B, dt, g, c, j)."""
    *lead, S, D = v.shape
    x = v.reshape(*lead, S // 32, 4, 8, D // 16, 16)
    n = len(lead)
    return x.permute(*range(n), n, n + 3, n + 1, n + 4, n + 2).contiguous().reshape(*lead, S * D)


def v_tiles_to_rows(vt, D):
    *lead, SD = vt.shape
    S = SD // D
    x = vt.reshape(*lead, S // 32, D // 16, 4, 16, 8)  # (B, dt, g, c, j)
    n = len(lead)
    return x.permute(*range(n), n, n + 2, n + 4, n + 1, n + 3).contiguous().reshape(*lead, S, D)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_ptr():
    import torch
    return torch.cuda.current_stream().cuda_stream


_LAYER_KEYS = ("wqkv", "wo", "w_gate_up", "w_down", "g_attn", "g_ffn")


def pack_matrix(w_bits):
    """Row-major int16 [N][K] device tensor -> streaming layout (device tensor of duo_packed_elems)."""
    import torch
    lib = load()
    N, K = w_bits.shape
    out = torch.empty(lib.duo_packed_elems(N, K), dtype=torch.int16, device=w_bits.device)
    _check(lib.duo_pack_matrix(w_bits.data_ptr(), N, K, out.data_ptr(), _stream_ptr()), "duo_pack_matrix")
    return out


def pack_activations(x_bits):
    import torch
    rows, K = x_bits.shape
    out = torch.empty((rows + 15) // 16 * 16 * K, dtype=torch.int16, device=x_bits.device)
    _check(load().duo_pack_activations(x_bits.data_ptr(), rows, K, out.data_ptr(), _stream_ptr()), "duo_pack_activations")
    return out


class DeviceWeights:
    """16-bit parameters (bf16 bit patterns as uint16 arrays, or numpy float16 arrays) on the GPU in the library's
    streaming layout (torch int16 tensors) + the C tables.  `dtype` is "bf16" or "fp16" accordingly.

    Row-major host matrices are uploaded one layer at a time, repacked on the device by the
    duo_pack_* entry points and dropped; only the packed copies stay resident.
    """

    def __init__(self, shape, host_weights: Dict[str, object], device: str = "cuda:0"):
        import torch
        lib = load()  # repacking moves 16-bit patterns: the same in both builds
        self.dtype = dtype_of(host_weights["embed"])
        cfg = make_config(shape, 32)
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device)
        empty = lambda n: torch.empty(n, dtype=torch.int16, device=device)
        sp = _stream_ptr()
        self.tensors: Dict[str, object] = {"embed": up(host_weights["embed"]), "g_final": up(host_weights["g_final"]),
                                           "lm_head": pack_matrix(up(host_weights["lm_head"]))}
        for key in _LAYER_KEYS:
            self.tensors[key] = []
        L = shape.n_layers
        for l in range(L):
            wq, wk, wv = (up(host_weights[k][l]) for k in ("wq", "wk", "wv"))
            qkv = empty(lib.duo_packed_elems(shape.q_dim + 2 * shape.kv_dim, shape.d_model))
            _check(lib.duo_pack_qkv(C.byref(cfg), wq.data_ptr(), wk.data_ptr(), wv.data_ptr(), qkv.data_ptr(), sp), "duo_pack_qkv")
            wg, wu = up(host_weights["w_gate"][l]), up(host_weights["w_up"][l])
            gu = empty(lib.duo_packed_elems(2 * shape.d_ff, shape.d_model))
            _check(lib.duo_pack_gate_up(C.byref(cfg), wg.data_ptr(), wu.data_ptr(), gu.data_ptr(), sp), "duo_pack_gate_up")
            self.tensors["wqkv"].append(qkv)
            self.tensors["w_gate_up"].append(gu)
            self.tensors["wo"].append(pack_matrix(up(host_weights["wo"][l])))
            self.tensors["w_down"].append(pack_matrix(up(host_weights["w_down"][l])))
            self.tensors["g_attn"].append(up(host_weights["g_attn"][l]))
            self.tensors["g_ffn"].append(up(host_weights["g_ffn"][l]))
            torch.cuda.synchronize()  # the row-major temporaries are released when this iteration ends
            del wq, wk, wv, wg, wu
        self.n_layers = L
        self._tables = {}
        self.c = Weights()
        self.c.embed = self.tensors["embed"].data_ptr()
        self.c.lm_head = self.tensors["lm_head"].data_ptr()
        self.c.g_final = self.tensors["g_final"].data_ptr()
        for key in _LAYER_KEYS:
            tab = (C.c_void_p * L)(*[t.data_ptr() for t in self.tensors[key]])
            self._tables[key] = tab
            setattr(self.c, key, C.cast(tab, C.POINTER(C.c_void_p)))


class VerifyEngine:
    """Owns the device buffers of one model instance (cache, workspace, results) and calls the C ABI."""

    def __init__(self, shape, host_weights: Dict[str, object], max_seq: int, device: str = "cuda:0",
                 max_rows: int = DUO_MAX_ROWS, weights: Optional[DeviceWeights] = None,
                 max_prefill_rows: int = DUO_MAX_ROWS):
        import torch
        self.torch = torch
        self.shape = shape
        self.device = device
        self.cfg = make_config(shape, max_seq)
        self.max_seq = max_seq
        self.weights = weights if weights is not None else DeviceWeights(shape, host_weights, device)
        self.dtype = self.weights.dtype   # the library build that matches the parameters' element type
        self.lib = load(self.dtype)
        L, H, D = shape.n_layers, shape.n_kv_heads, shape.head_dim
        # planes of max_seq * D elements in the library's tiled layouts (see k_rows_to_tiles / v_rows_to_tiles)
        self.k = torch.zeros((L, H, max_seq * D), dtype=torch.int16, device=device)
        self.vT = torch.zeros((L, H, max_seq * D), dtype=torch.int16, device=device)
        self.prefix_len = torch.zeros(1, dtype=torch.int32, device=device)
        self.root_logits = torch.zeros(shape.vocab, dtype=torch.float32, device=device)
        # verify calls take up to DUO_MAX_ROWS rows, prefill chunks up to DUO_MAX_PREFILL_ROWS (a larger workspace)
        self.max_prefill_rows = max(int(max_prefill_rows), min(int(max_rows), DUO_MAX_ROWS))
        self.ws_bytes = max(workspace_bytes(self.cfg, min(max_rows, DUO_MAX_ROWS)), workspace_bytes(self.cfg, self.max_prefill_rows))
        self.workspace = torch.zeros(self.ws_bytes, dtype=torch.uint8, device=device)
        self.accept_len = torch.zeros(DUO_MAX_ROWS, dtype=torch.int32, device=device)
        self.next_token = torch.zeros(DUO_MAX_ROWS, dtype=torch.int32, device=device)
        self.commit = torch.zeros(4, dtype=torch.int32, device=device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        self.cache_c = KVCache(self.k.data_ptr(), self.vT.data_ptr(), self.prefix_len.data_ptr(),
                               self.root_logits.data_ptr())
        self.host_prefix_len = 0

    # ---- cache management (plain copies, no arithmetic)
    def load_cache(self, k_bits: np.ndarray, v_bits: np.ndarray, prefix_len: int,
                   root_logits: Optional[np.ndarray]) -> None:
        """k_bits, v_bits: uint16 [L][Hkv][max_seq][D] (row layout); rearranged into the tiled layouts on upload."""
        torch = self.torch
        k = torch.from_numpy(np.ascontiguousarray(k_bits).view(np.int16)).to(self.device)
        self.k.copy_(k_rows_to_tiles(k).reshape(self.k.shape))
        del k
        v = torch.from_numpy(np.ascontiguousarray(v_bits).view(np.int16)).to(self.device)
        self.vT.copy_(v_rows_to_tiles(v).reshape(self.vT.shape))
        del v
        self.set_prefix_len(prefix_len)
        if root_logits is not None:
            self.root_logits.copy_(torch.from_numpy(np.asarray(root_logits, dtype=np.float32)))

    def set_prefix_len(self, p: int) -> None:
        self.host_prefix_len = int(p)
        self.prefix_len.fill_(int(p))

    def cache_to_host(self):
        """(k, v) as uint16 [L][Hkv][max_seq][D] in the row layout."""
        D = self.shape.head_dim
        host_type = np.float16 if self.dtype == "fp16" else np.uint16
        k = k_tiles_to_rows(self.k, D).cpu().numpy().view(host_type)
        v = v_tiles_to_rows(self.vT, D).cpu().numpy().view(host_type)
        return k, v

    # ---- entry points
    def prefill(self, tokens: Sequence[int], chunk: int = 64) -> None:
        torch = self.torch
        toks = torch.tensor(list(tokens), dtype=torch.int32, device=self.device)
        if chunk > self.max_prefill_rows:
            raise ValueError(f"prefill chunk {chunk} exceeds the engine's max_prefill_rows {self.max_prefill_rows}")
        for s in range(0, len(tokens), chunk):
            m = min(chunk, len(tokens) - s)
            rc = self.lib.duo_prefill_chunk(C.byref(self.cfg), C.byref(self.weights.c), C.byref(self.cache_c),
                                            toks[s:s + m].data_ptr(), m, self.host_prefix_len, self.status.data_ptr(),
                                            self.workspace.data_ptr(), self.ws_bytes, _stream_ptr())
            _check(rc, "duo_prefill_chunk")
            self.host_prefix_len += m

    def verify(self, draft_tokens, draft_probs, uniforms, temperature: float = 1.0,
               select_mode: int = SELECT_INDEPENDENT_LONGEST, root_token: int = -1, logits_out=None,
               top_p: float = 0.0) -> None:
        """Enqueue one verify step on torch's current stream.  Inputs are device tensors:
        draft_tokens int32 [n][k], draft_probs fp32 [n][k][V], uniforms fp32 [n][k+1]."""
        n, k = draft_tokens.shape
        call = Call(n, k, float(temperature), int(select_mode), int(root_token), self.host_prefix_len, float(top_p))
        res = Result(self.accept_len.data_ptr(), self.next_token.data_ptr(), self.commit.data_ptr(),
                     self.status.data_ptr(), _ptr(logits_out))
        rc = self.lib.duo_verify(C.byref(self.cfg), C.byref(self.weights.c), C.byref(self.cache_c),
                                 draft_tokens.data_ptr(), draft_probs.data_ptr(), uniforms.data_ptr(), C.byref(call),
                                 C.byref(res), self.workspace.data_ptr(), self.ws_bytes, _stream_ptr())
        _check(rc, "duo_verify")

    def verify_deferred(self, unverified_tokens, unverified_probs, uniforms, first_tokens=None, first_probs=None,
                        uniforms_first=None, temperature: float = 1.0, root_token: int = -1, logits_out=None,
                        top_p: float = 0.0) -> None:
        """Enqueue one round of Alg. 2 as listed (duo_verify_deferred) on torch's current stream.
        unverified_tokens int32 [l], unverified_probs fp32 [l][V], uniforms fp32 [l+1]; first_tokens int32 [s],
        first_probs fp32 [s][V], uniforms_first fp32 [s] (all three None for s = 0)."""
        l = 0 if unverified_tokens is None else int(unverified_tokens.shape[0])  # None: an empty suffix
        s_new = 0 if first_tokens is None else int(first_tokens.shape[0])
        call = Call(1, l, float(temperature), SELECT_PAPER_SEQUENTIAL, int(root_token), self.host_prefix_len, float(top_p))
        res = Result(self.accept_len.data_ptr(), self.next_token.data_ptr(), self.commit.data_ptr(),
                     self.status.data_ptr(), _ptr(logits_out))
        rc = self.lib.duo_verify_deferred(C.byref(self.cfg), C.byref(self.weights.c), C.byref(self.cache_c),
                                          _ptr(unverified_tokens) if l else None, _ptr(unverified_probs) if l else None,
                                          uniforms.data_ptr(),
                                          _ptr(first_tokens), _ptr(first_probs), _ptr(uniforms_first), s_new,
                                          C.byref(call), C.byref(res), self.workspace.data_ptr(), self.ws_bytes,
                                          _stream_ptr())
        _check(rc, "duo_verify_deferred")

    def results(self, n: int) -> Dict[str, object]:
        """Synchronise and fetch the outputs of the last verify call."""
        self.torch.cuda.synchronize()
        commit = self.commit.cpu().numpy()
        self.host_prefix_len = int(commit[3])  # the commit advanced the device-side prefix length
        return {"accept_len": self.accept_len[:n].cpu().numpy(), "next_token": self.next_token[:n].cpu().numpy(),
                "selected": int(commit[0]), "commit_len": int(commit[1]), "commit_token": int(commit[2]),
                "new_prefix_len": int(commit[3]), "status": int(self.status.cpu().numpy()[0]),
                "device_prefix_len": int(self.prefix_len.cpu().numpy()[0])}


def spec_sample(logits, root_logits, draft_tokens, draft_probs, uniforms, temperature: float = 1.0,
                select_mode: int = SELECT_INDEPENDENT_LONGEST, has_root: bool = False, prefix_len: int = 0,
                top_p: float = 0.0) -> Dict[str, object]:
    """duo_spec_sample on device tensors; returns host results."""
    import torch
    lib = load()
    n, k = draft_tokens.shape
    vocab = logits.shape[-1]
    nbytes = C.c_size_t(0)
    _check(lib.duo_sample_workspace_bytes(vocab, n, k, C.byref(nbytes)), "duo_sample_workspace_bytes")
    dev = logits.device
    ws = torch.empty(nbytes.value, dtype=torch.uint8, device=dev)
    accept_len = torch.zeros(n, dtype=torch.int32, device=dev)
    next_token = torch.zeros(n, dtype=torch.int32, device=dev)
    commit = torch.zeros(4, dtype=torch.int32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    call = Call(n, k, float(temperature), int(select_mode), 0 if has_root else -1, int(prefix_len), float(top_p))
    res = Result(accept_len.data_ptr(), next_token.data_ptr(), commit.data_ptr(), status.data_ptr(), None)
    rc = lib.duo_spec_sample(logits.data_ptr(), _ptr(root_logits), vocab, draft_tokens.data_ptr(), draft_probs.data_ptr(),
                             uniforms.data_ptr(), C.byref(call), C.byref(res), ws.data_ptr(), nbytes.value, _stream_ptr())
    _check(rc, "duo_spec_sample")
    torch.cuda.synchronize()
    c = commit.cpu().numpy()
    return {"accept_len": accept_len.cpu().numpy(), "next_token": next_token.cpu().numpy(), "selected": int(c[0]),
            "commit_len": int(c[1]), "commit_token": int(c[2]), "new_prefix_len": int(c[3]),
            "status": int(status.cpu().numpy()[0])}


class NoAllocSampler:
    """duo_spec_sample_noalloc with result buffers allocated once, here, by the caller: the call itself allocates
    nothing and takes no workspace.  Inputs are device tensors; `run` enqueues, `fetch` synchronises and reads."""

    def __init__(self, max_n: int = DUO_MAX_ROWS, device: str = "cuda:0"):
        import torch
        self.accept_len = torch.zeros(max_n, dtype=torch.int32, device=device)
        self.next_token = torch.zeros(max_n, dtype=torch.int32, device=device)
        self.commit = torch.zeros(4, dtype=torch.int32, device=device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)

    def run(self, logits, root_logits, draft_tokens, draft_probs, uniforms, temperature: float = 1.0,
            select_mode: int = SELECT_INDEPENDENT_LONGEST, has_root: bool = False, prefix_len: int = 0, top_p: float = 0.0,
            dtype: str = "bf16") -> int:
        """Returns the entry point's code (0 = enqueued) without raising, so that tests can look at error codes."""
        n, k = draft_tokens.shape
        vocab = logits.shape[-1]
        call = Call(n, k, float(temperature), int(select_mode), 0 if has_root else -1, int(prefix_len), float(top_p))
        res = Result(self.accept_len.data_ptr(), self.next_token.data_ptr(), self.commit.data_ptr(), self.status.data_ptr(), None)
        return int(load(dtype).duo_spec_sample_noalloc(logits.data_ptr(), _ptr(root_logits), vocab, draft_tokens.data_ptr(),
                                                       draft_probs.data_ptr(), uniforms.data_ptr(), C.byref(call), C.byref(res),
                                                       _stream_ptr()))

    def fetch(self, n: int) -> Dict[str, object]:
        import torch
        torch.cuda.synchronize()
        c = self.commit.cpu().numpy()
        return {"accept_len": self.accept_len[:n].cpu().numpy(), "next_token": self.next_token[:n].cpu().numpy(),
                "selected": int(c[0]), "commit_len": int(c[1]), "commit_token": int(c[2]), "new_prefix_len": int(c[3]),
                "status": int(self.status.cpu().numpy()[0])}


def deferred_sample(logits, root_logits, unverified_tokens, unverified_probs, uniforms, first_tokens=None,
                    first_probs=None, uniforms_first=None, temperature: float = 1.0, has_root: bool = False,
                    prefix_len: int = 0, top_p: float = 0.0) -> Dict[str, object]:
    """duo_deferred_sample on device tensors; returns host results.  An empty suffix: unverified_tokens None (logits then
    holds the root row only, or may be None without a root); `vocab` is then taken from root_logits."""
    import torch
    lib = load()
    l = 0 if unverified_tokens is None else int(unverified_tokens.shape[0])
    s_new = 0 if first_tokens is None else int(first_tokens.shape[0])
    vocab = (logits if logits is not None else root_logits).shape[-1]
    nbytes = C.c_size_t(0)
    _check(lib.duo_sample_workspace_bytes(vocab, 1, l, C.byref(nbytes)), "duo_sample_workspace_bytes")
    dev = (logits if logits is not None else root_logits).device
    ws = torch.empty(nbytes.value, dtype=torch.uint8, device=dev)
    accept_len = torch.zeros(1, dtype=torch.int32, device=dev)
    next_token = torch.zeros(1, dtype=torch.int32, device=dev)
    commit = torch.zeros(4, dtype=torch.int32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    call = Call(1, l, float(temperature), SELECT_PAPER_SEQUENTIAL, 0 if has_root else -1, int(prefix_len), float(top_p))
    res = Result(accept_len.data_ptr(), next_token.data_ptr(), commit.data_ptr(), status.data_ptr(), None)
    rc = lib.duo_deferred_sample(_ptr(logits), _ptr(root_logits), vocab, _ptr(unverified_tokens) if l else None,
                                 _ptr(unverified_probs) if l else None, uniforms.data_ptr(), _ptr(first_tokens), _ptr(first_probs),
                                 _ptr(uniforms_first), s_new, C.byref(call), C.byref(res), ws.data_ptr(), nbytes.value,
                                 _stream_ptr())
    _check(rc, "duo_deferred_sample")
    torch.cuda.synchronize()
    c = commit.cpu().numpy()
    return {"accept_len": int(accept_len.cpu().numpy()[0]), "next_token": int(next_token.cpu().numpy()[0]),
            "selected": int(c[0]), "commit_len": int(c[1]), "commit_token": int(c[2]), "new_prefix_len": int(c[3]),
            "status": int(status.cpu().numpy()[0])}


def skinny_gemm(x_bits, w_bits, dtype: str = "bf16"):
    """y = x W^T through duo_pack_activations / duo_pack_matrix / duo_skinny_gemm.
    x_bits int16 [rows][K], w_bits int16 [N][K] (row-major bf16 bit patterns on the device)."""
    import torch
    rows, K = x_bits.shape
    N = w_bits.shape[0]
    xp, wp = pack_activations(x_bits), pack_matrix(w_bits)
    y = torch.empty((rows, N), dtype=torch.float32, device=x_bits.device)
    _check(load(dtype).duo_skinny_gemm(xp.data_ptr(), wp.data_ptr(), y.data_ptr(), rows, N, K, _stream_ptr()), "duo_skinny_gemm")
    return y


def block_gemm(hi_bits, lo_bits, w_bits, dtype: str = "bf16"):
    """y = (hi + lo) W^T through duo_pack_activations / duo_pack_matrix / duo_block_gemm.
    hi_bits, lo_bits int16 [rows][K] (the two bf16 halves of the activations), w_bits int16 [N][K]."""
    import torch
    rows, K = hi_bits.shape
    N = w_bits.shape[0]
    pr = (rows + 15) // 16 * 16
    both = torch.zeros((2 * pr, K), dtype=torch.int16, device=hi_bits.device)
    both[:rows] = hi_bits
    both[pr:pr + rows] = lo_bits
    xp, wp = pack_activations(both), pack_matrix(w_bits)
    y = torch.empty((rows, N), dtype=torch.float32, device=hi_bits.device)
    _check(load(dtype).duo_block_gemm(xp.data_ptr(), wp.data_ptr(), y.data_ptr(), rows, N, K, _stream_ptr()), "duo_block_gemm")
    return y


def stream_read_probe(buf, sink, nontemporal: bool = False) -> None:
    """Enqueue one streaming read of the device tensor `buf` (duo_stream_read_probe), with ordinary loads or loads that
    carry the non-temporal hint; `sink` is an int32 tensor."""
    _check(load().duo_stream_read_probe(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), sink.numel(),
                                        1 if nontemporal else 0, _stream_ptr()), "duo_stream_read_probe")
