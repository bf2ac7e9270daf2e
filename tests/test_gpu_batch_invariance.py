"""With sled_model_set_batch_invariant the logits of a request are the same to the last bit whatever batch it is
verified in: alone, among requests with other draft lengths and context lengths, in a batch of more than 128 or
of more than 256 packed rows (where the default mode changes the projections' workgroup shape), and after its
context was built by prefill slices of different sizes.  Without the switch the same comparison shows the
round-off that the switch removes (reported, not asserted: it may happen to vanish)."""
import numpy as np
import pytest
import torch

from paper_2506_09397_amd import sled, synth
from paper_2506_09397_amd.runtime import Verifier

pytestmark = pytest.mark.gpu


def _probe_rows(v, shape, others_ctx, others_k, probe_ctx, probe_k, probe_tokens, seed):
    """Verify the probe request together with `others`; returns the probe's logits rows."""
    reqs, ks, toks = [], [], []
    rng = np.random.default_rng(seed)
    for L, k in zip(others_ctx, others_k):
        r = v.open()
        if L:
            K, V = synth.context_kv(shape, L, seed=seed, req=len(reqs) + 1, device="cuda")
            v.append_context([r], [K], [V])
        reqs.append(r); ks.append(k); toks.append(rng.integers(0, shape.vocab, size=k + 1).astype(np.int32))
    pos = len(reqs) // 2                       # the probe sits in the middle of the batch
    r = v.open()
    K, V = synth.context_kv(shape, probe_ctx, seed=99, req=0, device="cuda")
    v.append_context([r], [K], [V])
    reqs.insert(pos, r); ks.insert(pos, probe_k); toks.insert(pos, probe_tokens)
    logits = v.verify(reqs, ks, torch.from_numpy(np.concatenate(toks)).cuda())
    row0 = sum(k + 1 for k in ks[:pos])
    out = logits[row0: row0 + probe_k + 1].clone()
    torch.cuda.synchronize()
    for q in reqs:
        v.close_request(q)
    return out


BATCHES = [
    ([], []),                                                     # alone
    ([300, 40, 1000], [8, 0, 3]),                                 # a few others
    ([200] * 20, [5] * 20),                                       # 120 + rows: one block of rows
    ([64, 700, 16] * 12, [8, 2, 6] * 12),                         # > 256 rows, long and short contexts
]


@pytest.mark.parametrize("kind,layers", [("tiny_bf16", 0), ("llama8b", 2)])
def test_logits_do_not_depend_on_the_batch(kind, layers):
    shape = synth.SHAPES[kind]
    if layers:
        shape = synth.scaled_shape(shape, n_layers=layers, vocab=8192)
    w = synth.SynthWeights(shape, seed=3, device="cuda", std=0.05 if kind == "tiny_bf16" else 0.02)
    probe_ctx, probe_k = 1500, 6
    probe_tokens = np.random.default_rng(5).integers(0, shape.vocab, size=probe_k + 1).astype(np.int32)
    n_req = 40
    ctx_budget = probe_ctx + 36 * 780 + 64 * 9
    results = {}
    for invariant in (True, False):
        v = Verifier(shape, w, ctx_budget // 16 + 3 * n_req, n_req, n_req, ctx_budget, batch_invariant=invariant)
        rows = [_probe_rows(v, shape, c, k, probe_ctx, probe_k, probe_tokens, seed=7) for c, k in BATCHES]
        results[invariant] = rows
        v.destroy()
    worst = max(float((r - results[False][0]).abs().max()) for r in results[False][1:])
    print(f"{kind}: default mode, largest difference of the probe's logits between batchings: {worst:.3e}")
    for r in results[True][1:]:
        assert torch.equal(r, results[True][0])
    # and the two modes compute the same thing up to round-off
    assert float((results[True][0] - results[False][0]).abs().max()) < 5e-3


def test_prefill_slicing_does_not_change_the_cache_in_batch_invariant_mode():
    shape = synth.SHAPES["tiny_bf16"]
    w = synth.SynthWeights(shape, seed=4, device="cuda", std=0.05)
    prompt = torch.from_numpy(synth.context_tokens(333, shape.vocab, seed=8).astype(np.int32)).cuda()
    tail = torch.from_numpy(synth.context_tokens(5, shape.vocab, seed=9).astype(np.int32)).cuda()
    outs = []
    for b_max in (1, 4, 40):            # prefill slices of 9, 36 and 360 rows
        v = Verifier(shape, w, 64, 2, b_max, 1024, batch_invariant=True)
        r = v.open()
        last = v.prefill(r, prompt).clone()
        step = v.verify([r], [4], tail).clone()
        torch.cuda.synchronize()
        outs.append((last, step))
        v.destroy()
    for last, step in outs[1:]:
        assert torch.equal(last, outs[0][0]) and torch.equal(step, outs[0][1])
