"""GPU parity at full depth on the benchmark configurations (Sec. 3.1: one forward pass of the whole target over all
drafts; Sec. 3.4: one batch of heterogeneous requests): the library's logits against the oracle's, element by element.

  * Llama-3-8B shape, 32 layers, the batch of 16 that bench.py times: every row of every request;
  * the same model with the 64-request heterogeneous mix: four requests (the 8192-token one among them), then
    speculative-sampling acceptance over full-vocabulary draft probabilities on the library's own logits;
  * Llama-3-70B shape at its full 80 layers, batch of 32, one request scored, with the cache-rounding decisions taken
    as the library took them and audited (see the test).

These are the slow tests of the suite (the oracle widens every layer to float64): about six minutes together.
"""
import time

import numpy as np
import pytest
import torch

from oracle import sled_oracle as O
from paper_2506_09397_amd import sled, synth
from gpu_common import build_verifier, MARGIN_ACC, MARGIN_CDF
from helpers import oracle_model

# the oracle passes take minutes: these tests carry their own time limit, whatever --timeout the run was given
pytestmark = [pytest.mark.gpu, pytest.mark.slow, pytest.mark.timeout(600)]

TOL_BF16 = 2e-2


def _setup(shape, batch, seed, keep):
    B = batch.B
    ctx_budget = sum(batch.ctx_len) + 9 * B
    v, w = build_verifier(shape, seed, n_pages=ctx_budget // 16 + 2 * B + 8, max_requests=B, B_max=B,
                          ctx_tokens_max=ctx_budget)
    # contexts on physical pages scattered over the pool, as bench.py lays them out
    reqs = [v.open() for _ in range(B)]
    dev = [synth.context_kv(shape, batch.ctx_len[i], seed=seed, req=i, device="cuda") for i in range(B)]
    v.append_contexts_scattered(reqs, dev, seed=seed + 11)
    KV = {i: (dev[i][0].cpu(), dev[i][1].cpu()) for i in keep}
    del dev
    return v, w, reqs, KV


def _oracle_rows(shape, w, batch, KV, sample, round_points=None, say=None):
    """say: a function that prints past pytest's capture -- the oracle reports every fourth layer it has finished, so
    that a run of several minutes is seen to be alive."""
    offs = batch.row_offsets()
    oreqs = [{"tokens": batch.tokens[offs[i]: offs[i + 1]], "K": synth.as_f64(KV[i][0]), "V": synth.as_f64(KV[i][1])}
             for i in sample]
    t0 = time.time()
    def progress(l):
        if say is not None and (l % 4 == 3 or l + 1 == shape.n_layers):
            say(f"  oracle: layer {l + 1} of {shape.n_layers} done, {time.time() - t0:.0f} s")

    res = O.verify_batch(oracle_model(shape, w, round_points, cache=False), oreqs, progress)
    return [r["logits"] for r in res], time.time() - t0


@pytest.fixture
def say(capsys):
    def _say(msg):
        with capsys.disabled():
            print(msg, flush=True)
    return _say


def test_llama8b_b16_all_requests_32_layers(say):
    shape = synth.SHAPES["llama8b"]
    batch = synth.draw_batch("b16", shape.vocab, seed=0)
    say("\n8B shape, 32 layers, batch of 16: building the model")
    v, w, reqs, KV = _setup(shape, batch, 0, set(range(batch.B)))
    tokens = torch.from_numpy(batch.tokens).cuda()
    got = v.verify(reqs, batch.k, tokens).cpu().numpy()
    say("  library step done; oracle, all 16 requests")
    assert np.isfinite(got).all()
    offs = batch.row_offsets()
    want, dt = _oracle_rows(shape, w, batch, KV, list(range(batch.B)), say=say)
    errs = [float(np.abs(got[offs[i]: offs[i + 1]] - want[i]).max()) for i in range(batch.B)]
    say(f"8B, 32 layers, all {batch.B} requests (T={batch.T}): max |logit error| per request "
        f"{', '.join(f'{e:.1e}' for e in errs)}; worst {max(errs):.3e}; oracle {dt:.0f} s")
    assert max(errs) < TOL_BF16
    # how far the bf16 K/V cache alone moves the logits: the never-rounding oracle on two of the requests (reported,
    # and bounded loosely: it is a property of the model's storage, not of the kernels)
    pair = [int(np.argmax(batch.ctx_len)), int(np.argmin(batch.ctx_len))]
    exact, _ = _oracle_rows(shape, w, batch, KV, pair, "exact", say=say)
    d_def = max(float(np.abs(want[i] - e).max()) for i, e in zip(pair, exact))
    d_lib = max(float(np.abs(got[offs[i]: offs[i + 1]] - e).max()) for i, e in zip(pair, exact))
    say(f"never-rounding oracle at 32 layers (requests {pair}): the bf16-cache definition differs from it by {d_def:.3e}, "
        f"the library by {d_lib:.3e}")
    assert d_lib < d_def + TOL_BF16
    # greedy acceptance chained on the logits, wherever the oracle's top-2 gap is clear of the error
    a, t = v.accept(sled.GREEDY, batch.k, v.logits[: batch.T], tokens)
    acc = O.accept_batch("greedy", batch.k, np.concatenate(want).astype(np.float32).astype(np.float64), batch.tokens)
    a, t = a.cpu().numpy(), t.cpu().numpy()
    n = 0
    for i, r in enumerate(acc):
        if r["margin"] > 4 * max(errs):
            assert (a[i], t[i]) == (r["accept_len"], r["out_token"])
            n += 1
    assert n >= batch.B // 2
    v.destroy()


def test_llama8b_hetero64_32_layers_sampled_requests_and_sampling_acceptance(say):
    shape = synth.SHAPES["llama8b"]
    batch = synth.draw_batch("hetero64", shape.vocab, seed=0)
    order = np.argsort(batch.ctx_len)
    sample = sorted({int(order[-1]), int(order[0]), int(order[len(order) // 2]), int(order[3 * len(order) // 4])})
    assert max(batch.ctx_len[i] for i in sample) == max(batch.ctx_len) >= 7000      # the longest context of the mix
    say("\n8B shape, 32 layers, 64-request mix: building the model")
    v, w, reqs, KV = _setup(shape, batch, 0, set(sample))
    tokens = torch.from_numpy(batch.tokens).cuda()
    logits = v.verify(reqs, batch.k, tokens)
    got = logits.cpu().numpy()
    assert np.isfinite(got).all()
    offs = batch.row_offsets()
    want, dt = _oracle_rows(shape, w, batch, KV, sample, say=say)
    errs = [float(np.abs(got[offs[i]: offs[i + 1]] - r).max()) for i, r in zip(sample, want)]
    for i, e in zip(sample, errs):
        say(f"8B, 32 layers, hetero64 (T={batch.T}): request {i} (L={batch.ctx_len[i]}, k={batch.k[i]}): max |logit error| {e:.3e}")
    say(f"oracle time for {len(sample)} requests: {dt:.0f} s")
    assert max(errs) < TOL_BF16
    # speculative sampling (Eq. 1) over full-vocabulary draft probabilities on the library's own logits, all 64 requests
    nd = int(sum(batch.k))
    q = synth.draft_probs(nd, shape.vocab, 1.0, seed=3, device="cuda", base_std=1.28)
    u_acc = synth.uniforms(nd, seed=4, device="cuda")
    u_smp = synth.uniforms(batch.B, seed=5, device="cuda")
    a, t = v.accept(sled.SAMPLE, batch.k, logits, tokens, q, u_acc, u_smp)
    a, t = a.cpu().numpy(), t.cpu().numpy()
    ref = O.accept_batch("sample", batch.k, got.astype(np.float64), batch.tokens, synth.as_f64(q), synth.as_f64(u_acc),
                         synth.as_f64(u_smp))
    n_sub = 0
    for i, r in enumerate(ref):
        if r["margin_acc"] > MARGIN_ACC and r["margin_cdf"] > MARGIN_CDF:
            assert (int(a[i]), int(t[i])) == (r["accept_len"], r["out_token"]), f"request {i}"
        else:
            n_sub += 1
            assert 0 <= a[i] <= batch.k[i]
    assert n_sub <= 2
    v.commit(reqs, v.accept_len[: batch.B])
    assert v.lengths(reqs) == [L + int(x) + 1 for L, x in zip(batch.ctx_len, a)]
    v.destroy()


def test_llama70b_b32_80_layers_one_request(say):
    """Llama-3-70B shape at its full depth of 80 layers, the batch of 32 as benchmarked, one request scored.

    On this shape the rounding of new keys and values to the bf16 cache decides more than the tolerance: a value that
    the library computes (float32 sums) a hair to the other side of a rounding midpoint than the oracle (float64) is
    stored one bf16 step away, and a handful of such flips per layer move the final logits by 2e-2 and more -- for any
    implementation that does not reproduce the oracle's sums to the last bit (measured on the oracle itself: relative
    noise of 1e-5 on its projection outputs moves the logits of this shape by 3e-2 within 12 layers).  So the decision
    is taken as the library took it (the oracle attends to the numbers the library stored, read back through
    sled_kv_read) and audited: every stored number must be a correct rounding of a value within 1e-3 of its head
    vector's root mean square of the oracle's exact value (a twentieth of the relative tolerance on the logits).
    Everything else is the plain definition.  The error against the oracle left to its own rounding decisions is reported beside it."""
    shape = synth.SHAPES["llama70b"]
    batch = synth.draw_batch("b32", shape.vocab, seed=0)
    i = int(np.argsort(batch.ctx_len)[len(batch.ctx_len) // 2])
    say("\n70B shape, 80 layers, batch of 32: building the model (141 GB of weights)")
    v, w, reqs, KV = _setup(shape, batch, 0, {i})
    tokens = torch.from_numpy(batch.tokens).cuda()
    got = v.verify(reqs, batch.k, tokens).cpu().numpy()
    assert np.isfinite(got).all()
    n = batch.k[i] + 1
    Ks, Vs = v.read_kv(reqs[i], batch.ctx_len[i], n)          # the rows the step staged behind the context
    offs = batch.row_offsets()
    oreq = {"tokens": batch.tokens[offs[i]: offs[i + 1]], "K": synth.as_f64(KV[i][0]), "V": synth.as_f64(KV[i][1])}
    say("  library step done; oracle, 80 layers, attending to the numbers the library stored")
    t0 = time.time()

    def progress(l):
        if l % 8 == 7:
            say(f"  oracle: layer {l + 1} of {shape.n_layers} done, {time.time() - t0:.0f} s")

    om = oracle_model(shape, w, cache=False)
    res = O.verify_batch(om, [dict(oreq, K_stored=synth.as_f64(Ks), V_stored=synth.as_f64(Vs))], progress)[0]
    err = float(np.abs(got[offs[i]: offs[i + 1]] - res["logits"]).max())
    au = res["audit"]
    say(f"70B, 80 layers, b32 (T={batch.T}): request {i} (L={batch.ctx_len[i]}, k={batch.k[i]}): max |logit error| {err:.3e} "
        f"(logit std {res['logits'].std():.3f}); stored K/V: {au['flips']} of {au['elements']} differ from the oracle's own "
        f"rounding, worst {au['max_excess']:.2e} of the vector's rms beyond a correct rounding; oracle {time.time() - t0:.0f} s")
    assert au["max_excess"] < 1e-3
    assert err < TOL_BF16
    say("  oracle again, left to its own rounding decisions")
    plain = O.verify_batch(om, [oreq], progress)[0]
    err_plain = float(np.abs(got[offs[i]: offs[i + 1]] - plain["logits"]).max())
    say(f"  against the oracle's own rounding decisions: max |logit error| {err_plain:.3e}")
    assert err_plain < 0.25          # sanity only: this distance is the flips' doing, see above
    v.destroy()
