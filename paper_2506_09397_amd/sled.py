"""ctypes binding of libsled.so -- argument marshalling only.

Every function has the name and the meaning of the C entry point declared in
include/sled.h; tensors are torch tensors on the GPU (device memory and streams are
all PyTorch is used for), per-request integers are Python sequences.  Errors raise
SledError.  There is no fallback: if the library has not been built, importing the
symbols fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

from .synth import ModelShape

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsled.so")

OK, EINVAL, ENOMEM, ESTATE, EHIP = 0, -1, -2, -3, -4
F32, BF16 = 0, 1
GREEDY, SAMPLE = 0, 1
T_EMBED, T_WQ, T_WK, T_WV, T_WO, T_WGATE, T_WUP, T_WDOWN, T_G_ATTN, T_G_MLP, T_G_FINAL, T_LM_HEAD = range(12)
T_SCALE = 100   # + a matrix id: that matrix's per-row scales (models with 8-bit weights)
TENSOR_IDS = {"embed": T_EMBED, "wq": T_WQ, "wk": T_WK, "wv": T_WV, "wo": T_WO, "wg": T_WGATE, "wu": T_WUP,
              "wd": T_WDOWN, "g_attn": T_G_ATTN, "g_mlp": T_G_MLP, "g_final": T_G_FINAL, "lm_head": T_LM_HEAD}

EXPORTS = [
    "sled_model_create", "sled_model_load", "sled_model_destroy", "sled_model_set_batch_invariant",
    "sled_model_set_weight_bits",
    "sled_kvpool_create", "sled_kvpool_open", "sled_kvpool_close", "sled_kvpool_lengths", "sled_kvpool_destroy",
    "sled_kv_append", "sled_kv_read", "sled_verify_workspace_bytes", "sled_verify_batch", "sled_prefill",
    "sled_attention_partition", "sled_projection_slices",
    "sled_accept_workspace_bytes", "sled_accept", "sled_accept_static", "sled_accept_sparse", "sled_row_confidence", "sled_profile_enable", "sled_profile_read",
    "sled_strerror", "sled_last_error",
]
PROF_PROJ, PROF_ATTN, PROF_ROWS, PROF_N = 0, 1, 2, 3


class SledError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"sled error {code}: {msg}")
        self.code = code


class _Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab",
                                           "dtype")] + [("rms_eps", C.c_float), ("rope_theta", C.c_float),
                                                        ("page_size", C.c_int32), ("k_max", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """Loads libsled.so (built by paper_2506_09397_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not found: run `python -m paper_2506_09397_amd.build` (hipcc, gfx950)")
    L = C.CDLL(LIB_PATH)
    vp, ip = C.c_void_p, C.POINTER(C.c_int)
    L.sled_model_create.argtypes = [C.POINTER(_Shape), C.POINTER(vp)]
    L.sled_model_load.argtypes = [vp, C.c_int, C.c_int, vp, vp]
    L.sled_model_destroy.argtypes = [vp]
    L.sled_model_set_batch_invariant.argtypes = [vp, C.c_int]
    L.sled_model_set_weight_bits.argtypes = [vp, C.c_int]
    L.sled_kvpool_create.argtypes = [vp, C.c_int64, C.c_int, C.POINTER(vp)]
    L.sled_kvpool_open.argtypes = [vp, ip]
    L.sled_kvpool_close.argtypes = [vp, C.c_int]
    L.sled_kvpool_lengths.argtypes = [vp, C.c_int, ip, ip, vp]
    L.sled_kvpool_destroy.argtypes = [vp]
    L.sled_kv_append.argtypes = [vp, C.c_int, ip, ip, C.POINTER(vp), C.POINTER(vp), vp, vp]
    L.sled_kv_read.argtypes = [vp, C.c_int, C.c_int, C.c_int, vp, vp, vp]
    L.sled_verify_workspace_bytes.argtypes = [vp, C.c_int, C.c_int, C.c_int64]
    L.sled_attention_partition.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int)]
    L.sled_projection_slices.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
    L.sled_verify_workspace_bytes.restype = C.c_size_t
    L.sled_verify_batch.argtypes = [vp, vp, C.c_int, ip, ip, vp, vp, vp, C.c_size_t, vp]
    L.sled_prefill.argtypes = [vp, vp, C.c_int, C.c_int, vp, vp, vp, C.c_size_t, vp]
    L.sled_accept_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int]
    L.sled_accept_workspace_bytes.restype = C.c_size_t
    L.sled_accept.argtypes = [C.c_int, C.c_int, ip, C.c_int, C.c_float, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    L.sled_accept_static.argtypes = [C.c_int, C.c_int, ip, C.c_int, C.c_float, vp, vp, vp, vp, vp, vp, vp, vp]
    L.sled_accept_sparse.argtypes = [C.c_int, ip, C.c_int, C.c_float, vp, vp, C.c_int, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    L.sled_row_confidence.argtypes = [C.c_int, C.c_int, C.c_float, vp, vp, vp, vp, C.c_size_t, vp]
    L.sled_profile_enable.argtypes = [vp, C.c_int]
    L.sled_profile_read.argtypes = [vp, vp, C.POINTER(C.c_float), ip]
    L.sled_strerror.argtypes = [C.c_int]
    L.sled_strerror.restype = C.c_char_p
    L.sled_last_error.restype = C.c_char_p
    for name in EXPORTS:
        getattr(L, name)  # AttributeError here means the library is stale: rebuild it
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != OK:
        L = lib()
        raise SledError(rc, f"{L.sled_strerror(rc).decode()}: {L.sled_last_error().decode()}")


def _ints(xs: Sequence[int]):
    return (C.c_int * len(xs))(*[int(x) for x in xs])


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device pointers must come from contiguous CUDA tensors"
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


# ---------------------------------------------------------------------------------------- model
def sled_model_create(shape: ModelShape) -> int:
    s = _Shape(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
               shape.vocab, F32 if shape.dtype == "f32" else BF16, shape.rms_eps, shape.rope_theta, shape.page_size,
               shape.k_max)
    h = C.c_void_p()
    _check(lib().sled_model_create(C.byref(s), C.byref(h)))
    return h.value


def sled_model_load(model: int, tensor_id: int, layer: int, src: torch.Tensor) -> None:
    _check(lib().sled_model_load(model, tensor_id, layer, _ptr(src), _stream()))


def sled_model_destroy(model: int) -> None:
    _check(lib().sled_model_destroy(model))


# ---------------------------------------------------------------------------------------- pool
def sled_kvpool_create(model: int, n_pages: int, max_requests: int) -> int:
    h = C.c_void_p()
    _check(lib().sled_kvpool_create(model, n_pages, max_requests, C.byref(h)))
    return h.value


def sled_kvpool_open(pool: int) -> int:
    r = C.c_int(-1)
    _check(lib().sled_kvpool_open(pool, C.byref(r)))
    return r.value


def sled_kvpool_close(pool: int, req_id: int) -> None:
    _check(lib().sled_kvpool_close(pool, req_id))


def sled_kvpool_lengths(pool: int, req_ids: Sequence[int]):
    out = (C.c_int * len(req_ids))()
    _check(lib().sled_kvpool_lengths(pool, len(req_ids), _ints(req_ids), out, _stream()))
    return list(out)


def sled_kvpool_destroy(pool: int) -> None:
    _check(lib().sled_kvpool_destroy(pool))


def sled_kv_append(pool: int, req_ids: Sequence[int], n_tokens: Optional[Sequence[int]] = None,
                   k_src: Optional[Sequence[torch.Tensor]] = None, v_src: Optional[Sequence[torch.Tensor]] = None,
                   accept_len: Optional[torch.Tensor] = None) -> None:
    B = len(req_ids)
    if accept_len is not None:
        assert accept_len.dtype == torch.int32
        _check(lib().sled_kv_append(pool, B, _ints(req_ids), None, None, None, _ptr(accept_len), _stream()))
        return
    kp = (C.c_void_p * B)(*[_ptr(t) for t in k_src])
    vp = (C.c_void_p * B)(*[_ptr(t) for t in v_src])
    _check(lib().sled_kv_append(pool, B, _ints(req_ids), _ints(n_tokens), kp, vp, None, _stream()))


def sled_kv_read(pool: int, req_id: int, first_token: int, n_tokens: int, k_dst: torch.Tensor, v_dst: torch.Tensor) -> None:
    _check(lib().sled_kv_read(pool, int(req_id), int(first_token), int(n_tokens), _ptr(k_dst), _ptr(v_dst), _stream()))


# ---------------------------------------------------------------------------------------- step
def sled_verify_workspace_bytes(model: int, B_max: int, T_max: int, ctx_tokens_max: int) -> int:
    return int(lib().sled_verify_workspace_bytes(model, B_max, T_max, ctx_tokens_max))


def sled_attention_partition(n_kv_heads: int, n_pages: Sequence[int]):
    """(pages per attention work item, number of work items) for a step over requests holding n_pages[i] pages."""
    a, b = C.c_int(0), C.c_int(0)
    _check(lib().sled_attention_partition(n_kv_heads, len(n_pages), _ints(n_pages), C.byref(a), C.byref(b)))
    return a.value, b.value


def sled_projection_slices(n_out: int, n_in: int, T: int):
    """(K slices in a step of T rows, the most a step may use) for a projection n_in -> n_out of a bf16 model."""
    a, b = C.c_int(0), C.c_int(0)
    _check(lib().sled_projection_slices(n_out, n_in, T, C.byref(a), C.byref(b)))
    return a.value, b.value


def sled_verify_batch(model: int, pool: int, req_ids: Sequence[int], k: Sequence[int], tokens: torch.Tensor,
                      logits: torch.Tensor, workspace: torch.Tensor) -> None:
    assert tokens.dtype == torch.int32 and logits.dtype == torch.float32
    _check(lib().sled_verify_batch(model, pool, len(req_ids), _ints(req_ids), _ints(k), _ptr(tokens), _ptr(logits),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def sled_prefill(model: int, pool: int, req_id: int, tokens: torch.Tensor, logits_last: Optional[torch.Tensor],
                 workspace: torch.Tensor) -> None:
    assert tokens.dtype == torch.int32 and (logits_last is None or logits_last.dtype == torch.float32)
    _check(lib().sled_prefill(model, pool, int(req_id), int(tokens.numel()), _ptr(tokens), _ptr(logits_last), _ptr(workspace),
                              workspace.numel() * workspace.element_size(), _stream()))


def sled_accept_workspace_bytes(B: int, T: int, vocab: int) -> int:
    return int(lib().sled_accept_workspace_bytes(B, T, vocab))


def sled_accept(mode: int, k: Sequence[int], vocab: int, temperature: float, logits: torch.Tensor, tokens: torch.Tensor,
                draft_q: Optional[torch.Tensor], u_acc: Optional[torch.Tensor], u_smp: Optional[torch.Tensor],
                accept_len: torch.Tensor, out_token: torch.Tensor, workspace: torch.Tensor) -> None:
    assert logits.dtype == torch.float32 and tokens.dtype == torch.int32
    assert accept_len.dtype == torch.int32 and out_token.dtype == torch.int32
    _check(lib().sled_accept(mode, len(k), _ints(k), vocab, float(temperature), _ptr(logits), _ptr(tokens), _ptr(draft_q),
                             _ptr(u_acc), _ptr(u_smp), _ptr(accept_len), _ptr(out_token), _ptr(workspace),
                             workspace.numel() * workspace.element_size(), _stream()))


def sled_accept_static(mode: int, k: Sequence[int], vocab: int, temperature: float, logits: torch.Tensor, tokens: torch.Tensor,
                       draft_q: Optional[torch.Tensor], u_acc: Optional[torch.Tensor], u_smp: Optional[torch.Tensor],
                       accept_len: torch.Tensor, out_token: torch.Tensor) -> None:
    assert logits.dtype == torch.float32 and tokens.dtype == torch.int32
    assert accept_len.dtype == torch.int32 and out_token.dtype == torch.int32
    _check(lib().sled_accept_static(mode, len(k), _ints(k), vocab, float(temperature), _ptr(logits), _ptr(tokens),
                                    _ptr(draft_q), _ptr(u_acc), _ptr(u_smp), _ptr(accept_len), _ptr(out_token), _stream()))


def sled_accept_sparse(k: Sequence[int], vocab: int, temperature: float, logits: torch.Tensor, tokens: torch.Tensor,
                       q_ids: torch.Tensor, q_probs: torch.Tensor, u_acc: torch.Tensor, u_smp: torch.Tensor,
                       accept_len: torch.Tensor, out_token: torch.Tensor, workspace: torch.Tensor,
                       q_rest: Optional[torch.Tensor] = None) -> None:
    assert logits.dtype == torch.float32 and tokens.dtype == torch.int32
    assert q_ids.dtype == torch.int32 and q_probs.dtype == torch.float32 and q_ids.shape == q_probs.shape
    assert q_rest is None or (q_rest.dtype == torch.float32 and q_rest.numel() == q_ids.shape[0])
    _check(lib().sled_accept_sparse(len(k), _ints(k), vocab, float(temperature), _ptr(logits), _ptr(tokens), int(q_ids.shape[-1]),
                                    _ptr(q_ids), _ptr(q_probs), _ptr(q_rest), _ptr(u_acc), _ptr(u_smp), _ptr(accept_len), _ptr(out_token),
                                    _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def sled_row_confidence(vocab: int, temperature: float, logits: torch.Tensor, conf: torch.Tensor, top: Optional[torch.Tensor],
                        workspace: torch.Tensor) -> None:
    assert logits.dtype == torch.float32 and conf.dtype == torch.float32 and (top is None or top.dtype == torch.int32)
    _check(lib().sled_row_confidence(int(logits.shape[0]), vocab, float(temperature), _ptr(logits), _ptr(conf),
                                     _ptr(top) if top is not None else None, _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream()))


def sled_model_set_batch_invariant(model: int, on: bool) -> None:
    _check(lib().sled_model_set_batch_invariant(model, 1 if on else 0))


def sled_profile_enable(model: int, on: bool) -> None:
    _check(lib().sled_profile_enable(model, 1 if on else 0))


def sled_profile_read(model: int):
    ms = (C.c_float * PROF_N)()
    n = (C.c_int * PROF_N)()
    _check(lib().sled_profile_read(model, _stream(), ms, n))
    return list(ms), list(n)


# ---------------------------------------------------------------------------------------- helpers
def load_weights(model: int, weights) -> None:
    """Streams every tensor of a synth.SynthWeights-like object (on the GPU) into the model.  An object with
    bits == 8 (synth.SynthWeightsW8) is loaded as FP8 bytes plus per-row scales, one with bits == 4
    (synth.SynthWeightsW4) as packed FP4 codes plus block exponents."""
    bits = getattr(weights, "bits", 16)
    w8 = bits != 16
    if weights.shape.dtype == "bf16":
        _check(lib().sled_model_set_weight_bits(model, bits))   # also back to 16 on a model that held another format

    def put(name: str, layer: int) -> None:
        if w8 and name in weights.MATRICES:
            sled_model_load(model, TENSOR_IDS[name], layer, weights.q(name, layer).contiguous().view(torch.uint8))
            sled_model_load(model, T_SCALE + TENSOR_IDS[name], layer, weights.scale(name, layer).contiguous())
        else:
            sled_model_load(model, TENSOR_IDS[name], layer, weights.tensor(name, layer).contiguous())

    sled_model_load(model, T_EMBED, 0, weights.embed().contiguous())
    for l in range(weights.shape.n_layers):
        for name in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g_attn", "g_mlp"):
            put(name, l)
    for name in ("g_final", "lm_head"):
        put(name, -1)
    torch.cuda.synchronize()


def workspace(n_bytes: int) -> torch.Tensor:
    """Device scratch of n_bytes, 256-byte aligned (torch's allocator aligns to 512)."""
    return torch.empty((n_bytes + 255) // 256 * 256, dtype=torch.uint8, device="cuda")
