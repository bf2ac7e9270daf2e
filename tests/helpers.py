"""Glue used by the tests only: turns seeded synthetic inputs into what the oracle takes."""
from __future__ import annotations

import numpy as np

from oracle import sled_oracle as O
from paper_2506_09397_amd import synth


class F64Weights:
    """float64 numpy view of synth.SynthWeights (exact widening), cached for small models."""

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

    def layer(self, l):
        return self._get(("layer", l), lambda: {k: synth.as_f64(v) for k, v in self.w.layer(l).items()})

    def final(self):
        return self._get("final", lambda: {k: synth.as_f64(v) for k, v in self.w.final().items()})


def oracle_model(shape: synth.ModelShape, weights: synth.SynthWeights, round_points=None, cache=True) -> O.OracleModel:
    if round_points is None:
        round_points = "bf16" if shape.dtype == "bf16" else "exact"
    return O.OracleModel(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                         shape.d_ffn, shape.vocab, shape.rope_theta, shape.rms_eps,
                         F64Weights(weights, cache), round_points)


def split_rows(batch: synth.Batch, arr: np.ndarray):
    offs = batch.row_offsets()
    return [arr[offs[i]: offs[i + 1]] for i in range(batch.B)]
