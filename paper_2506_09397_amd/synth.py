"""Seeded synthetic inputs for batched speculative verification.

This module only *draws inputs*: model shapes, random weights, ragged batches of
verification requests, context K/V, draft distributions and uniforms.  It holds
none of the method's arithmetic (no transformer layer, no attention, no acceptance
rule) and is shared by the tests of the CPU oracle and of the HIP library, so that
both see identical values.  Everything is a function of an integer seed.

Workload shapes follow the paper's setting: many edge devices, each with its own
context length and its own speculative length, send draft tokens that one shared
LLaMA-family target model verifies in a batch (Sec. 3.2, Sec. 3.4, Sec. 4).  The
paper publishes no request traces, so lengths are drawn from simple seeded
distributions (uniform, log-uniform, a four-point mix of speculative lengths).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import numpy as np
import torch


# --------------------------------------------------------------------------- shapes
@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Architecture constants of a LLaMA-family decoder (Sec. 4 names the family only)."""

    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str  # "f32" or "bf16": storage type of weights, activations fed to GEMMs, and K/V
    rope_theta: float
    rms_eps: float = 1e-5
    page_size: int = 16
    k_max: int = 8

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def layer_params(self) -> int:
        d, hq, hkv, D, F = self.d_model, self.n_q_heads, self.n_kv_heads, self.head_dim, self.d_ffn
        return d * hq * D + 2 * d * hkv * D + hq * D * d + 3 * d * F

    def streamed_params(self) -> int:
        """Parameters every verify step must read once: all layers plus the LM head."""
        return self.n_layers * self.layer_params() + self.vocab * self.d_model

    def kv_bytes_per_token(self) -> int:
        esz = 4 if self.dtype == "f32" else 2
        return 2 * self.n_kv_heads * self.head_dim * esz * self.n_layers


SHAPES: Dict[str, ModelShape] = {
    # 2-layer fp32 decoder, no GQA
    "tiny": ModelShape(2, 256, 4, 4, 64, 1024, 1024, "f32", 10000.0),
    # same, bf16 storage, with GQA: exercises the bf16 kernels at a size the oracle finishes fast
    "tiny_bf16": ModelShape(2, 256, 8, 2, 128, 1024, 1024, "bf16", 10000.0),
    # Llama-3-8B-shaped
    "llama8b": ModelShape(32, 4096, 32, 8, 128, 14336, 128256, "bf16", 500000.0),
    # Llama-3-70B-shaped
    "llama70b": ModelShape(80, 8192, 64, 8, 128, 28672, 128256, "bf16", 500000.0),
}


def scaled_shape(base: ModelShape, **kw) -> ModelShape:
    return dataclasses.replace(base, **kw)


# --------------------------------------------------------------------------- weights
_TENSOR_IDS = {
    "embed": 0, "wq": 1, "wk": 2, "wv": 3, "wo": 4, "wg": 5, "wu": 6, "wd": 7,
    "g_attn": 8, "g_mlp": 9, "g_final": 10, "lm_head": 11,
}


def _seed_for(seed: int, tensor: str, layer: int) -> int:
    return (seed * 1_000_003 + _TENSOR_IDS[tensor] * 10_007 + (layer + 1) * 101) % (2**31 - 1)


class SynthWeights:
    """Random-init weights N(0, std) in the model's storage dtype; norm gains 1 (+ optional jitter).

    Linear weights use the [out_features, in_features] convention: y = x @ W.T.
    Every tensor is regenerated on demand from (seed, tensor name, layer), so a model
    far larger than host memory can be streamed layer by layer.
    """

    def __init__(self, shape: ModelShape, seed: int = 0, device: str = "cpu",
                 std: float = 0.02, gain_jitter: float = 0.0):
        self.shape, self.seed, self.device, self.std, self.gain_jitter = shape, seed, device, std, gain_jitter

    def _randn(self, tensor: str, layer: int, *size: int) -> torch.Tensor:
        g = torch.Generator(device=self.device)
        g.manual_seed(_seed_for(self.seed, tensor, layer))
        return torch.randn(*size, generator=g, device=self.device, dtype=torch.float32)

    def _mat(self, tensor: str, layer: int, out_f: int, in_f: int) -> torch.Tensor:
        return (self._randn(tensor, layer, out_f, in_f) * self.std).to(self.shape.torch_dtype)

    def _gain(self, tensor: str, layer: int) -> torch.Tensor:
        g = torch.ones(self.shape.d_model, device=self.device, dtype=torch.float32)
        if self.gain_jitter:
            g = g + self.gain_jitter * self._randn(tensor, layer, self.shape.d_model)
        return g.to(self.shape.torch_dtype)

    def embed(self) -> torch.Tensor:
        return self._mat("embed", -1, self.shape.vocab, self.shape.d_model)

    def tensor(self, name: str, layer: int = -1) -> torch.Tensor:
        s = self.shape
        dims = {
            "wq": (s.n_q_heads * s.head_dim, s.d_model), "wk": (s.n_kv_heads * s.head_dim, s.d_model),
            "wv": (s.n_kv_heads * s.head_dim, s.d_model), "wo": (s.d_model, s.n_q_heads * s.head_dim),
            "wg": (s.d_ffn, s.d_model), "wu": (s.d_ffn, s.d_model), "wd": (s.d_model, s.d_ffn),
            "lm_head": (s.vocab, s.d_model), "embed": (s.vocab, s.d_model),
        }
        if name in dims:
            return self._mat(name, layer, *dims[name])
        return self._gain(name, layer)

    def layer(self, l: int) -> Dict[str, torch.Tensor]:
        return {n: self.tensor(n, l) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g_attn", "g_mlp")}

    def final(self) -> Dict[str, torch.Tensor]:
        return {"g_final": self.tensor("g_final"), "lm_head": self.tensor("lm_head")}


class SynthWeightsW8(SynthWeights):
    """The same model with 8-bit projection weights: the stored numbers are one byte per weight (an OCP FP8 E4M3
    code, the encoding torch calls float8_e4m3fn) and one scale per output row.  The bytes are drawn the way a
    quantiser would produce them -- N(0, 16) rounded to the nearest FP8 number -- and the scales as
    bf16-representable values around std / 16, so that the matrix the bytes stand for has entries of standard
    deviation about std.  Bytes and scales are the *inputs* of both the HIP library and the CPU oracle; what they
    mean (the float matrix) is decoded by each side on its own, never here.

    q() returns the bytes, uint8 [out, in]; scale() the float32 row scales [out].  Embedding and gains as in
    SynthWeights (tensor() serves only those)."""

    bits = 8
    MATRICES = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "lm_head")

    def q(self, name: str, layer: int = -1) -> torch.Tensor:
        out_f, in_f = self._dims()[name]
        z = torch.clamp(self._randn(name, layer, out_f, in_f) * 16.0, -240.0, 240.0)
        return z.to(torch.float8_e4m3fn).view(torch.uint8)   # the quantiser's rounding; only the bytes leave

    def scale(self, name: str, layer: int = -1) -> torch.Tensor:
        out_f, _ = self._dims()[name]
        g = torch.Generator(device=self.device)
        g.manual_seed((_seed_for(self.seed, name, layer) * 7 + 13) % (2**31 - 1))
        u = torch.rand(out_f, generator=g, device=self.device, dtype=torch.float32)
        return ((self.std / 16.0) * (0.75 + 0.5 * u)).to(torch.bfloat16).to(torch.float32)

    def _dims(self):
        s = self.shape
        return {
            "wq": (s.n_q_heads * s.head_dim, s.d_model), "wk": (s.n_kv_heads * s.head_dim, s.d_model),
            "wv": (s.n_kv_heads * s.head_dim, s.d_model), "wo": (s.d_model, s.n_q_heads * s.head_dim),
            "wg": (s.d_ffn, s.d_model), "wu": (s.d_ffn, s.d_model), "wd": (s.d_model, s.d_ffn),
            "lm_head": (s.vocab, s.d_model),
        }

    def tensor(self, name: str, layer: int = -1) -> torch.Tensor:
        if name in self.MATRICES:
            raise TypeError(f"{name}: a low-bit matrix exists only as codes and scales (q(), scale()); "
                            "what they mean is for the consumer to decode")
        return SynthWeights.tensor(self, name, layer)

    def layer(self, l: int):
        raise TypeError("low-bit weights have no float layer(): use q() / scale() per matrix")

    def final(self):
        raise TypeError("low-bit weights have no float final(): use q() / scale() per matrix")


class SynthWeightsW4(SynthWeightsW8):
    """The same model with 4-bit projection weights in the microscaling arrangement: a 4-bit code per weight, two
    per byte, and one scale byte per output row and block of 32 inputs.  Codes and scale bytes are drawn the way a
    quantiser would produce them from an N(0, std) matrix -- the block's scale is the smallest power of two that
    brings its largest magnitude within the code range (6), each scaled weight goes to the nearest of the eight
    code magnitudes -- and, as for 8 bits, they are inputs: decoding them is the consumer's business.

    q() returns the packed codes, uint8 [out, in / 2], even input index in the low nibble, bit 3 of a code the
    sign; scale() the scale bytes (biased exponent, bias 127), uint8 [out, in / 32]."""

    bits = 4
    _LEVELS = (0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0)   # quantiser's output levels, code = index (+ 8 if negative)

    def _codes(self, name: str, layer: int):
        out_f, in_f = self._dims()[name]
        w = self._randn(name, layer, out_f, in_f) * self.std
        blocks = w.view(out_f, in_f // 32, 32)
        amax = blocks.abs().amax(dim=2).clamp_min(1e-30)
        e = torch.ceil(torch.log2(amax / 6.0)).clamp(-100, 100)           # smallest power of two with amax / 2^e <= 6
        x = torch.ldexp(blocks, (-e).to(torch.int32)[:, :, None])
        levels = torch.tensor(self._LEVELS, device=w.device, dtype=torch.float32)
        mid = (levels[1:] + levels[:-1]) / 2
        mag = torch.bucketize(x.abs().contiguous(), mid)                  # index of the nearest level
        code = (mag + 8 * (x < 0)).to(torch.uint8).view(out_f, in_f)
        return code, (e + 127).to(torch.uint8)

    def q(self, name: str, layer: int = -1) -> torch.Tensor:
        code, _ = self._codes(name, layer)
        return (code[:, 0::2] | (code[:, 1::2] << 4)).contiguous()

    def scale(self, name: str, layer: int = -1) -> torch.Tensor:
        return self._codes(name, layer)[1].contiguous()


def as_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a stored tensor (fp32 or bf16) to a float64 numpy array on the host."""
    return t.detach().to("cpu").to(torch.float64).numpy()


# --------------------------------------------------------------------------- batches
@dataclasses.dataclass
class Batch:
    """A ragged batch of verification requests.

    ctx_len[i]  context tokens of request i already in the KV cache
    k[i]        number of draft tokens of request i
    tokens      packed int32 [sum(k)+B]: for each request [pending token, draft_1..draft_k]
    """

    ctx_len: List[int]
    k: List[int]
    tokens: np.ndarray

    @property
    def B(self) -> int:
        return len(self.k)

    @property
    def T(self) -> int:
        return int(sum(self.k)) + len(self.k)

    def row_offsets(self) -> List[int]:
        off, out = 0, []
        for ki in self.k:
            out.append(off)
            off += ki + 1
        out.append(off)
        return out


def draw_batch(kind: str, vocab: int, seed: int = 0, B: Optional[int] = None) -> Batch:
    """Draw request lengths for one of the named traffic mixes.

    "tiny4"     4 requests, 64 context tokens, k = 4
    "b16"       16 requests, context uniform in [512, 2048], k uniform in [2, 8]
    "hetero64"  64 requests, context log-uniform in [128, 8192], k in {2,4,6,8} w.p. {.4,.3,.2,.1}
                (stands in for a fleet of unequal devices with unequal speculative lengths)
    "b32"       32 requests, context uniform in [1024, 4096], k uniform in [4, 8]
    Integer ranges are inclusive at both ends.
    """
    rng = np.random.default_rng(seed)
    if kind == "tiny4":
        B = B or 4
        L = [64] * B
        k = [4] * B
    elif kind == "b16":
        B = B or 16
        L = rng.integers(512, 2049, size=B).tolist()
        k = rng.integers(2, 9, size=B).tolist()
    elif kind == "hetero64":
        B = B or 64
        L = np.clip(np.rint(np.exp(rng.uniform(math.log(128), math.log(8192), size=B))), 128, 8192)
        L = L.astype(np.int64).tolist()
        k = rng.choice([2, 4, 6, 8], size=B, p=[0.4, 0.3, 0.2, 0.1]).tolist()
    elif kind == "b32":
        B = B or 32
        L = rng.integers(1024, 4097, size=B).tolist()
        k = rng.integers(4, 9, size=B).tolist()
    else:
        raise ValueError(kind)
    T = int(sum(k)) + B
    tokens = rng.integers(0, vocab, size=T).astype(np.int32)
    return Batch([int(x) for x in L], [int(x) for x in k], tokens)


def make_batch(ctx_len: List[int], k: List[int], vocab: int, seed: int = 0) -> Batch:
    rng = np.random.default_rng(seed)
    T = int(sum(k)) + len(k)
    return Batch(list(ctx_len), list(k), rng.integers(0, vocab, size=T).astype(np.int32))


def context_tokens(n: int, vocab: int, seed: int) -> np.ndarray:
    return np.random.default_rng(seed + 7919).integers(0, vocab, size=n).astype(np.int32)


def context_kv(shape: ModelShape, n_tokens: int, seed: int, req: int, device: str = "cpu"):
    """Context K (taken as already rotated) and V ~ N(0,1) in the storage dtype,
    each [n_layers, n_tokens, n_kv_heads, head_dim]."""
    g = torch.Generator(device=device)
    g.manual_seed((seed * 7_368_787 + req * 50_021 + 17) % (2**31 - 1))
    size = (shape.n_layers, n_tokens, shape.n_kv_heads, shape.head_dim)
    K = torch.randn(size, generator=g, device=device, dtype=torch.float32).to(shape.torch_dtype)
    V = torch.randn(size, generator=g, device=device, dtype=torch.float32).to(shape.torch_dtype)
    return K, V


# --------------------------------------------------------------------------- acceptance inputs
@dataclasses.dataclass
class AcceptCase:
    """Inputs of the acceptance step alone.

    logits  fp32 [T, V] target logits, rows packed per request (k_i + 1 rows each)
    tokens  int32 [T]   [pending, draft_1..draft_k] per request
    q       fp32 [sum k, V] draft probabilities, one row per draft token, request-major
    u_acc   fp32 [sum k]   uniforms in [0,1) for the accept tests
    u_smp   fp32 [B]       uniforms in [0,1) for the single resample / bonus draw
    """

    k: List[int]
    logits: torch.Tensor
    tokens: torch.Tensor
    q: torch.Tensor
    u_acc: torch.Tensor
    u_smp: torch.Tensor


def accept_case(k: List[int], vocab: int, sigma: float, seed: int = 0, device: str = "cpu",
                target_std: float = 2.0, drafts_from_q: bool = True) -> AcceptCase:
    """Target logits z ~ N(0, target_std); the draft distribution of draft j is
    softmax(z_row + sigma * N(0,1)) where z_row is the target row that judges it; draft
    ids are drawn from that distribution (or uniformly when drafts_from_q is False)."""
    g = torch.Generator(device=device)
    g.manual_seed((seed * 2_654_435 + 12345) % (2**31 - 1))
    B, T, nd = len(k), sum(k) + len(k), sum(k)
    logits = torch.randn(T, vocab, generator=g, device=device, dtype=torch.float32) * target_std
    judge_rows = []
    off = 0
    for ki in k:
        judge_rows += list(range(off, off + ki))
        off += ki + 1
    idx = torch.tensor(judge_rows, device=device, dtype=torch.long)
    q = torch.empty(nd, vocab, device=device, dtype=torch.float32)
    drafts = torch.empty(nd, device=device, dtype=torch.long)
    step = 256
    for s in range(0, nd, step):
        sl = slice(s, min(nd, s + step))
        zl = logits[idx[sl]] + sigma * torch.randn(idx[sl].numel(), vocab, generator=g, device=device,
                                                    dtype=torch.float32)
        q[sl] = torch.softmax(zl, dim=-1)
        if drafts_from_q:
            drafts[sl] = torch.multinomial(q[sl], 1, generator=g).squeeze(1)
        else:
            drafts[sl] = torch.randint(0, vocab, (idx[sl].numel(),), generator=g, device=device)
    tokens = torch.empty(T, device=device, dtype=torch.int32)
    off = doff = 0
    pend = torch.randint(0, vocab, (B,), generator=g, device=device)
    for i, ki in enumerate(k):
        tokens[off] = pend[i]
        tokens[off + 1: off + 1 + ki] = drafts[doff: doff + ki].to(torch.int32)
        off += ki + 1
        doff += ki
    u_acc = torch.rand(nd, generator=g, device=device, dtype=torch.float32)
    u_smp = torch.rand(B, generator=g, device=device, dtype=torch.float32)
    return AcceptCase(list(k), logits, tokens, q, u_acc, u_smp)


def draft_probs(n_rows: int, vocab: int, noise: float, seed: int, device: str = "cpu",
                base_std: float = 1.0) -> torch.Tensor:
    """Draft probabilities softmax(z + noise * eps), z ~ N(0, base_std), eps ~ N(0,1), fp32 [n_rows, vocab]."""
    g = torch.Generator(device=device)
    g.manual_seed((seed * 97_003 + 4242) % (2**31 - 1))
    out = torch.empty(n_rows, vocab, device=device, dtype=torch.float32)
    step = 256
    for s in range(0, n_rows, step):
        n = min(step, n_rows - s)
        z = base_std * torch.randn(n, vocab, generator=g, device=device, dtype=torch.float32)
        e = torch.randn(n, vocab, generator=g, device=device, dtype=torch.float32)
        out[s:s + n] = torch.softmax(z + noise * e, dim=-1)
    return out


def uniforms(n: int, seed: int, device: str = "cpu") -> torch.Tensor:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 31_337 + 99) % (2**31 - 1))
    return torch.rand(n, generator=g, device=device, dtype=torch.float32)
