"""Models with 8-bit and 4-bit projection weights (weight-only quantisation, the 8- and 4-bit points of the
bit-width sweep of Sec. 4.3): the library loads FP8 E4M3 bytes and their per-row scales, or FP4 E2M1 codes and
their block exponents; the oracle multiplies with the dequantised matrices in float64.  Same storage contract
for activations, same tolerance as for bf16 weights."""
import numpy as np
import pytest
import torch

from oracle import sled_oracle as O
from paper_2506_09397_amd import sled, synth
from paper_2506_09397_amd.runtime import Verifier
from helpers import oracle_model, oracle_requests

pytestmark = pytest.mark.gpu


def _run(shape, w, ctx_len, k, seed, tol, batch_invariant=False):
    B = len(k)
    budget = sum(ctx_len) + 9 * B
    v = Verifier(shape, w, budget // 16 + 3 * B + 8, B, B, budget, batch_invariant=batch_invariant)
    batch = synth.make_batch(ctx_len, k, shape.vocab, seed=seed)
    reqs = [v.open() for _ in range(B)]
    Ks, Vs = [], []
    for i in range(B):
        K, V = synth.context_kv(shape, ctx_len[i], seed=seed, req=i, device="cuda")
        Ks.append(K); Vs.append(V)
    v.append_context(reqs, Ks, Vs)
    tokens = torch.from_numpy(batch.tokens).cuda()
    got = v.verify(reqs, k, tokens).cpu().numpy().astype(np.float64)
    want = np.concatenate([r["logits"] for r in O.verify_batch(oracle_model(shape, w), oracle_requests(batch, Ks, Vs))], axis=0)
    err = np.abs(got - want).max()
    print(f"{w.bits}-bit weights, B={B} T={batch.T}: max |logit error| = {err:.3e} (logit std {want.std():.3f})")
    assert err < tol
    # greedy acceptance on these logits equals the oracle's on its own
    a, t = v.accept(sled.GREEDY, k, torch.from_numpy(got.astype(np.float32)).cuda(), tokens)
    ref = O.accept_batch("greedy", k, got.astype(np.float32).astype(np.float64), batch.tokens)
    assert a.cpu().tolist() == [r["accept_len"] for r in ref] and t.cpu().tolist() == [r["out_token"] for r in ref]
    v.destroy()


@pytest.mark.parametrize("ctx_len,k", [
    ([64, 64, 64, 64], [4, 4, 4, 4]),
    ([0, 5, 16, 17, 130, 257, 1000], [8, 0, 3, 8, 1, 7, 8]),
    ([300] * 20, [2, 4, 6, 8] * 5),            # 120 rows: one full block
    ([90] * 15, [8] * 15),                     # 135 rows: the wide shape
    ([200, 40, 333] * 15, [8, 7, 8] * 15),     # 390 rows
])
def test_tiny_model_with_8bit_weights(ctx_len, k):
    shape = synth.SHAPES["tiny_bf16"]
    w = synth.SynthWeightsW8(shape, seed=2, device="cuda", std=0.02, gain_jitter=0.1)
    _run(shape, w, ctx_len, k, seed=4, tol=5e-3)


def test_8b_shape_two_layers_with_8bit_weights():
    shape = synth.scaled_shape(synth.SHAPES["llama8b"], n_layers=2, vocab=8192)
    w = synth.SynthWeightsW8(shape, seed=1, device="cuda")
    _run(shape, w, [700, 33, 1500, 256, 90], [8, 2, 5, 0, 7], seed=6, tol=2e-2)


@pytest.mark.parametrize("ctx_len,k", [
    ([64, 64, 64, 64], [4, 4, 4, 4]),
    ([0, 5, 16, 17, 130, 257, 1000], [8, 0, 3, 8, 1, 7, 8]),
    ([300] * 20, [2, 4, 6, 8] * 5),            # 120 rows: one full block
    ([90] * 15, [8] * 15),                     # 135 rows: the wide shape
    ([200, 40, 333] * 15, [8, 7, 8] * 15),     # 390 rows
])
def test_tiny_model_with_4bit_weights(ctx_len, k):
    shape = synth.SHAPES["tiny_bf16"]
    w = synth.SynthWeightsW4(shape, seed=2, device="cuda", std=0.02, gain_jitter=0.1)
    _run(shape, w, ctx_len, k, seed=4, tol=5e-3)


def test_8b_shape_two_layers_with_4bit_weights():
    shape = synth.scaled_shape(synth.SHAPES["llama8b"], n_layers=2, vocab=8192)
    w = synth.SynthWeightsW4(shape, seed=1, device="cuda")
    _run(shape, w, [700, 33, 1500, 256, 90], [8, 2, 5, 0, 7], seed=6, tol=2e-2)


@pytest.mark.parametrize("cls", [synth.SynthWeightsW8, synth.SynthWeightsW4])
def test_full_vocabulary_head_with_lowbit_weights(cls):
    """104 rows and the full 128256-token vocabulary: the LM head runs in its 512-column shape (no K groups), where
    the 4-bit scale blocks advance by half a block per stage."""
    shape = synth.scaled_shape(synth.SHAPES["llama8b"], n_layers=1)
    w = cls(shape, seed=5, device="cuda")
    _run(shape, w, [40] * 13, [7] * 13, seed=8, tol=2e-2)


@pytest.mark.parametrize("cls", [synth.SynthWeightsW8, synth.SynthWeightsW4])
def test_lowbit_weights_in_batch_invariant_mode(cls):
    """390 rows with the batch-invariant switch: three row blocks through the narrow projection shape."""
    shape = synth.SHAPES["tiny_bf16"]
    w = cls(shape, seed=2, device="cuda", std=0.02, gain_jitter=0.1)
    _run(shape, w, [200, 40, 333] * 15, [8, 7, 8] * 15, seed=4, tol=5e-3, batch_invariant=True)


@pytest.mark.parametrize("cls", [synth.SynthWeightsW8, synth.SynthWeightsW4])
def test_prompt_ingest_with_lowbit_weights(cls):
    """sled_prefill on a model with 8- or 4-bit weights: many-row slices (the wide projection shape) and the one-row
    LM head, against the oracle's plain causal forward over the prompt."""
    shape = synth.SHAPES["tiny_bf16"]
    w = cls(shape, seed=6, device="cuda", std=0.05, gain_jitter=0.1)
    v = Verifier(shape, w, 64, 2, 40, 1024)
    om = oracle_model(shape, w)
    for L in (9, 300):
        p = synth.context_tokens(L, shape.vocab, seed=70 + L)
        r = v.open()
        got = v.prefill(r, torch.from_numpy(p.astype(np.int32)).cuda()).cpu().numpy().astype(np.float64)
        err = np.abs(got - O.prefill(om, p)["logits"][-1]).max()
        print(f"{w.bits}-bit weights, prompt of {L}: max |last-token logit error| = {err:.3e}")
        assert err < 5e-3 and v.lengths([r]) == [L]
    v.destroy()


def test_one_model_reloaded_in_every_weight_format():
    """sled_model_set_weight_bits gives the matrices' storage back and allocates it anew for the next format: the
    same model handle loaded with 8-bit, 4-bit and 16-bit weights in turn matches the oracle each time."""
    shape = synth.SHAPES["tiny_bf16"]
    ctx_len, k = [33, 200, 0], [5, 8, 2]
    B = len(k)
    v = Verifier(shape, synth.SynthWeightsW8(shape, seed=2, device="cuda", gain_jitter=0.1), 64, B, B, 512)
    batch = synth.make_batch(ctx_len, k, shape.vocab, seed=9)
    reqs = [v.open() for _ in range(B)]
    Ks, Vs = [], []
    for i in range(B):
        K, V = synth.context_kv(shape, ctx_len[i], seed=9, req=i, device="cuda")
        Ks.append(K); Vs.append(V)
    v.append_context(reqs, Ks, Vs)
    tokens = torch.from_numpy(batch.tokens).cuda()
    for cls in (synth.SynthWeightsW8, synth.SynthWeightsW4, synth.SynthWeights, synth.SynthWeightsW4):
        w = cls(shape, seed=2, device="cuda", gain_jitter=0.1)
        sled.load_weights(v.model, w)
        got = v.verify(reqs, k, tokens).cpu().numpy().astype(np.float64)
        want = np.concatenate([r["logits"] for r in O.verify_batch(oracle_model(shape, w), oracle_requests(batch, Ks, Vs))], axis=0)
        err = np.abs(got - want).max()
        print(f"{getattr(w, 'bits', 16)}-bit weights on the reused model: max |logit error| = {err:.3e}")
        assert err < 5e-3
    v.destroy()


def test_weight_bits_argument_errors():
    shape = synth.SHAPES["tiny"]                # an fp32 model cannot take 8-bit weights
    m = sled.sled_model_create(shape)
    with pytest.raises(sled.SledError):
        sled._check(sled.lib().sled_model_set_weight_bits(m, 8))
    sled.sled_model_destroy(m)
    m = sled.sled_model_create(synth.SHAPES["tiny_bf16"])
    with pytest.raises(sled.SledError):
        sled._check(sled.lib().sled_model_set_weight_bits(m, 2))
    with pytest.raises(sled.SledError):          # scales for a 16-bit model
        sled.sled_model_load(m, sled.T_SCALE + sled.T_WQ, 0, torch.ones(1024, device="cuda"))
    sled.sled_model_destroy(m)
