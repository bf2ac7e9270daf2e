"""Glue between the seeded input generators and the oracle (test infrastructure, like the oracle).

Turns synth.SynthWeights (torch tensors in the model's storage type, on any device) into the
float64 numpy accessors sled_oracle.OracleModel takes.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np

from oracle import lowbit
from oracle import sled_oracle as O
from paper_2506_09397_amd import synth   # seeded input generators only: no arithmetic of the method lives there

_LAYER_MATS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd")


class F64Weights:
    """float64 numpy view of synth.SynthWeights (exact widening); cached when asked (small models,
    or a few layers of a large one).  Low-bit weights (bits 8 or 4) arrive as codes and scales and are
    decoded here by oracle.lowbit, from the format definitions."""

    def __init__(self, w: synth.SynthWeights, cache: bool = True):
        self.w, self.cache, self._c = w, cache, {}

    def _get(self, key, fn):
        if not self.cache:
            return fn()
        if key not in self._c:
            self._c[key] = fn()
        return self._c[key]

    def embed(self):
        return self._get("embed", lambda: synth.as_f64(self.w.embed()))

    def _matrix(self, name, l):
        bits = getattr(self.w, "bits", 16)
        if bits == 16:
            return synth.as_f64(self.w.tensor(name, l))
        q, sc = self.w.q(name, l).cpu().numpy(), self.w.scale(name, l).cpu().numpy()
        return lowbit.dequant_fp8_rows(q, sc) if bits == 8 else lowbit.dequant_mxfp4(q, sc)

    def _layer(self, l):
        out = {n: self._matrix(n, l) for n in _LAYER_MATS}
        for n in ("g_attn", "g_mlp"):
            out[n] = synth.as_f64(self.w.tensor(n, l))
        return out

    def layer(self, l):
        return self._get(("layer", l), lambda: self._layer(l))

    def final(self):
        return self._get("final", lambda: {"g_final": synth.as_f64(self.w.tensor("g_final")),
                                           "lm_head": self._matrix("lm_head", -1)})


def oracle_model(shape: synth.ModelShape, weights: synth.SynthWeights, round_points=None, cache=True,
                 n_layers=None) -> O.OracleModel:
    """round_points defaults to the definition for the model's dtype: "kv_bf16" (exact arithmetic over a
    bf16 K/V cache) for a bf16 model, "exact" for an fp32 one.  n_layers < shape.n_layers
    gives the oracle for the first n_layers layers followed by the final norm and LM head."""
    if round_points is None:
        round_points = "kv_bf16" if shape.dtype == "bf16" else "exact"
    return O.OracleModel(shape.n_layers if n_layers is None else n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                         shape.d_ffn, shape.vocab, shape.rope_theta, shape.rms_eps, F64Weights(weights, cache),
                         round_points)


def oracle_requests(batch: synth.Batch, K_list, V_list, n_layers=None):
    reqs, offs = [], batch.row_offsets()
    for i in range(batch.B):
        K, V = K_list[i], V_list[i]
        if n_layers is not None:
            K, V = K[:n_layers], V[:n_layers]
        reqs.append({"tokens": batch.tokens[offs[i]: offs[i + 1]], "K": synth.as_f64(K), "V": synth.as_f64(V)})
    return reqs
