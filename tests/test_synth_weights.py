"""The synthetic low-bit weights are inputs to both sides; this checks on the host that the matrix the oracle
multiplies with is exactly what the stored numbers mean under the format's definition."""
import numpy as np

from paper_2506_09397_amd import synth


def test_4bit_synthetic_weights_mean_what_they_say():
    """The dequantised matrix handed to the oracle is the stored codes and exponents decoded by the format's
    definition (checked here value by value on the host), it stays close to the N(0, std) draw it was rounded
    from, and every block exponent is the smallest that keeps the block within the code range."""
    shape = synth.SHAPES["tiny_bf16"]
    w = synth.SynthWeightsW4(shape, seed=3, device="cpu")
    q, e, t = w.q("wd", 1).numpy(), w.scale("wd", 1).numpy(), w.tensor("wd", 1).numpy()
    mags = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    rng = np.random.default_rng(0)
    for _ in range(2000):
        n, k = int(rng.integers(t.shape[0])), int(rng.integers(t.shape[1]))
        code = (int(q[n, k // 2]) >> (4 * (k & 1))) & 15
        val = (-1.0 if code & 8 else 1.0) * mags[code & 7] * 2.0 ** (int(e[n, k // 32]) - 127)
        assert t[n, k] == np.float32(val)
    assert 1 <= e.min() and e.max() <= 254
    assert 0.8 * w.std < t.std() < 1.2 * w.std
    top = np.abs(t).reshape(t.shape[0], -1, 32).max(axis=2) / 2.0 ** (e.astype(np.float64) - 127)
    assert (top >= 3.0).all() and (top <= 6.0).all()      # amax / 2^e lies in (3, 6] before rounding


def test_8bit_synthetic_weights_mean_what_they_say():
    """FP8 E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities) decoded from the bytes by
    hand equals the matrix handed to the oracle."""
    shape = synth.SHAPES["tiny_bf16"]
    w = synth.SynthWeightsW8(shape, seed=3, device="cpu")
    import torch
    q = w.q("wo", 0).view(torch.uint8).numpy()
    sc, t = w.scale("wo", 0).numpy(), w.tensor("wo", 0).numpy()
    rng = np.random.default_rng(1)
    for _ in range(2000):
        n, k = int(rng.integers(t.shape[0])), int(rng.integers(t.shape[1]))
        b = int(q[n, k])
        sign, ex, man = -1.0 if b & 0x80 else 1.0, (b >> 3) & 15, b & 7
        val = sign * (man / 8.0 * 2.0 ** -6 if ex == 0 else (1 + man / 8.0) * 2.0 ** (ex - 7))
        assert t[n, k] == np.float32(np.float32(val) * sc[n])
