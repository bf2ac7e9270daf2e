"""The synthetic low-bit weights are inputs to both sides: the generator draws codes and scales, the oracle decodes
them (oracle/lowbit.py, pinned in test_oracle_lowbit.py).  This checks on the host that the draws are what a
quantiser would produce -- block exponents minimal, magnitudes in range, matrix statistics as intended -- and that
the generator module itself decodes nothing."""
import numpy as np
import pytest
import torch

from helpers import F64Weights
from paper_2506_09397_amd import synth


def test_4bit_synthetic_weights_mean_what_they_say():
    shape = synth.SHAPES["tiny_bf16"]
    w = synth.SynthWeightsW4(shape, seed=3, device="cpu")
    q, e = w.q("wd", 1).numpy(), w.scale("wd", 1).numpy()
    t = F64Weights(w).layer(1)["wd"]
    mags = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    rng = np.random.default_rng(0)
    for _ in range(2000):   # the matrix the oracle multiplies with, decoded by hand from the stored numbers
        n, k = int(rng.integers(t.shape[0])), int(rng.integers(t.shape[1]))
        code = (int(q[n, k // 2]) >> (4 * (k & 1))) & 15
        val = (-1.0 if code & 8 else 1.0) * mags[code & 7] * 2.0 ** (int(e[n, k // 32]) - 127)
        assert t[n, k] == val
    assert 1 <= e.min() and e.max() <= 254
    assert 0.8 * w.std < t.std() < 1.2 * w.std
    top = np.abs(t).reshape(t.shape[0], -1, 32).max(axis=2) / 2.0 ** (e.astype(np.float64) - 127)
    assert (top >= 3.0).all() and (top <= 6.0).all()      # amax / 2^e lies in (3, 6] before rounding


def test_8bit_synthetic_weights_mean_what_they_say():
    shape = synth.SHAPES["tiny_bf16"]
    w = synth.SynthWeightsW8(shape, seed=3, device="cpu")
    q = w.q("wo", 0).numpy()
    assert q.dtype == np.uint8 and not ((q & 0x7F) == 0x7F).any()     # bytes, none of them the NaN pattern
    sc = w.scale("wo", 0).numpy()
    t = F64Weights(w).layer(0)["wo"]
    rng = np.random.default_rng(1)
    for _ in range(2000):
        n, k = int(rng.integers(t.shape[0])), int(rng.integers(t.shape[1]))
        b = int(q[n, k])
        sign, ex, man = -1.0 if b & 0x80 else 1.0, (b >> 3) & 15, b & 7
        val = sign * (man / 8.0 * 2.0 ** -6 if ex == 0 else (1 + man / 8.0) * 2.0 ** (ex - 7))
        assert t[n, k] == val * float(sc[n])
    assert 0.8 * w.std < t.std() < 1.2 * w.std
    assert np.array_equal(sc, torch.from_numpy(sc).to(torch.bfloat16).to(torch.float32).numpy())   # bf16-representable


@pytest.mark.parametrize("cls", [synth.SynthWeightsW8, synth.SynthWeightsW4])
def test_generator_hands_out_codes_not_matrices(cls):
    w = cls(synth.SHAPES["tiny_bf16"], seed=0, device="cpu")
    with pytest.raises(TypeError):
        w.tensor("wq", 0)
    with pytest.raises(TypeError):
        w.layer(0)
    assert w.tensor("g_attn", 0).shape == (synth.SHAPES["tiny_bf16"].d_model,)
