"""Host-side state of the K/V pool around the step (Sec. 3.2's rounds, Sec. 3.3's retries): page accounting between a
verify and its commit, prompt ingest of a new request while another batch awaits its commit, partial commits,
requests opened into recycled slots, and the asynchronous tightening of the page bounds.  Values are checked against
the oracle where a wrong state would corrupt cached K/V."""
import numpy as np
import pytest
import torch

from oracle import sled_oracle as O
from paper_2506_09397_amd import sled, synth
from paper_2506_09397_amd.runtime import Verifier
from helpers import oracle_model

pytestmark = pytest.mark.gpu


def _tiny(n_pages=64, max_requests=6):
    shape = synth.SHAPES["tiny"]
    w = synth.SynthWeights(shape, seed=4, device="cuda", std=0.05, gain_jitter=0.1)
    v = Verifier(shape, w, n_pages, max_requests, max_requests, 16 * n_pages)
    return shape, w, v, oracle_model(shape, w)


def _dev(x):
    return torch.tensor(x, dtype=torch.int32, device="cuda")


def test_lengths_between_verify_and_commit_keeps_the_staged_pages():
    """verify -> lengths -> commit -> verify: the rows staged at positions L .. L+k sit on a page the committed length
    does not reach yet; asking for the lengths in between must not hand that page to somebody else."""
    shape, w, v, om = _tiny(n_pages=8, max_requests=3)
    prompt = synth.context_tokens(14, shape.vocab, seed=1)          # 14 cached tokens: rows 14..22 spill onto page 1
    r = v.open()
    v.prefill(r, _dev(prompt), want_logits=False)
    drafts = [int(t) for t in synth.context_tokens(9, shape.vocab, seed=2)]
    v.verify([r], [8], _dev(drafts))
    assert v.lengths([r]) == [14]                                    # the sync in the middle
    # another request now takes pages: it must not get the one that holds the staged rows
    r2 = v.open()
    v.prefill(r2, _dev(synth.context_tokens(40, shape.vocab, seed=3)), want_logits=False)
    v.commit([r], _dev([8]))                                         # all 9 staged rows become context
    assert v.lengths([r, r2]) == [23, 40]
    nxt = [int(t) for t in synth.context_tokens(3, shape.vocab, seed=5)]
    got = v.verify([r], [2], _dev(nxt)).cpu().numpy()
    pf = O.prefill(om, list(prompt) + drafts)
    want = O.verify_batch(om, [{"tokens": nxt, "K": pf["K"], "V": pf["V"]}])[0]["logits"]
    assert np.abs(got - want).max() < 1e-4
    v.destroy()


def test_prefill_of_a_new_request_does_not_break_a_pending_commit():
    shape, w, v, om = _tiny()
    ctx = [synth.context_tokens(20 + 7 * i, shape.vocab, seed=10 + i) for i in range(2)]
    reqs = [v.open() for _ in ctx]
    for r, c in zip(reqs, ctx):
        v.prefill(r, _dev(c), want_logits=False)
    toks = [int(t) for t in synth.context_tokens(8, shape.vocab, seed=30)]
    v.verify(reqs, [3, 3], _dev(toks))
    newcomer = v.open()                                              # a new device's prompt arrives before the commit
    v.prefill(newcomer, _dev(synth.context_tokens(33, shape.vocab, seed=31)), want_logits=False)
    v.commit(reqs, _dev([3, 1]))
    assert v.lengths(reqs + [newcomer]) == [24, 29, 33]
    # a prefill of a request that HAS staged rows overwrites them: that request alone loses its commit
    v.verify(reqs, [2, 2], _dev(toks[:6]))
    v.prefill(reqs[0], _dev(synth.context_tokens(5, shape.vocab, seed=32)), want_logits=False)
    with pytest.raises(sled.SledError) as e:
        v.commit(reqs, _dev([2, 2]))
    assert e.value.code == sled.ESTATE
    v.commit([reqs[1]], _dev([0]))                                   # the other one still can, on its own
    assert v.lengths(reqs) == [29, 30]
    with pytest.raises(sled.SledError):
        v.commit([reqs[1]], _dev([0]))                               # ... but only once
    v.destroy()


def test_recycled_slot_starts_empty_and_open_close_do_not_wait():
    """A request opened into a slot that held a longer one starts at length 0 although open() enqueues nothing."""
    shape, w, v, om = _tiny(n_pages=16, max_requests=2)
    a = v.open()
    v.prefill(a, _dev(synth.context_tokens(50, shape.vocab, seed=40)), want_logits=False)
    v.close_request(a)
    b = v.open()
    assert b == a and v.lengths([b]) == [0]
    prompt = synth.context_tokens(11, shape.vocab, seed=41)
    got = v.prefill(b, _dev(prompt)).cpu().numpy()
    want = O.prefill(om, prompt)["logits"][-1]
    assert np.abs(got - want).max() < 1e-4
    assert v.lengths([b]) == [11]
    v.destroy()


def test_page_bounds_tighten_without_a_sync():
    """Commits that accept nothing: the host first has to assume all 9 staged rows were kept, so a pool this small
    would run out of pages within a few rounds; the exact lengths that follow every commit back to the host let it
    go on for many rounds with no call that waits."""
    shape, w, v, om = _tiny(n_pages=6, max_requests=2)
    r = v.open()
    v.prefill(r, _dev(synth.context_tokens(10, shape.vocab, seed=50)), want_logits=False)
    toks = _dev([int(t) for t in synth.context_tokens(9, shape.vocab, seed=51)])
    zero = _dev([0])
    for step in range(40):                                           # 40 x 9 staged rows would need 23 pages
        v.verify([r], [8], toks)
        v.commit([r], zero)                                          # one token per round is kept
        if step % 4 == 3:
            torch.cuda.current_stream().synchronize()                # time passes (the copies land); no pool call waits
    assert v.lengths([r]) == [50]
    v.destroy()


@pytest.mark.parametrize("kind", ["tiny", "tiny_bf16"])
def test_kv_read_returns_what_append_and_verify_wrote(kind):
    """sled_kv_read against both ways in: context appended from outside comes back bit for bit, and the rows a verify
    stages are the oracle's new K/V (float32 model: to round-off; bf16 model: the same bf16 numbers, up to a rare
    value that sits within round-off of a rounding midpoint and is stored one step away)."""
    shape = synth.SHAPES[kind]
    w = synth.SynthWeights(shape, seed=8, device="cuda", std=0.05, gain_jitter=0.1)
    v = Verifier(shape, w, 32, 2, 2, 256)
    om = oracle_model(shape, w)
    L = 21
    K, V = synth.context_kv(shape, L, seed=3, req=0, device="cuda")
    r = v.open()
    v.append_context([r], [K], [V])
    Kb, Vb = v.read_kv(r, 0, L)
    assert torch.equal(Kb, K) and torch.equal(Vb, V)
    Kb, Vb = v.read_kv(r, 5, 9)
    assert torch.equal(Kb, K[:, 5:14]) and torch.equal(Vb, V[:, 5:14])
    toks = [int(t) for t in synth.context_tokens(7, shape.vocab, seed=4)]
    v.verify([r], [6], _dev(toks))
    Kn, Vn = v.read_kv(r, L, 7)
    req = {"tokens": toks, "K": synth.as_f64(K), "V": synth.as_f64(V)}
    if kind == "tiny":
        want = O.verify_batch(om, [req])[0]
        assert np.abs(synth.as_f64(Kn) - want["K_new"]).max() < 1e-5 and np.abs(synth.as_f64(Vn) - want["V_new"]).max() < 1e-5
    else:
        # every stored number is a correct rounding of a value within 1e-4 of its head vector's rms of what the oracle
        # computes when it attends to the same stored numbers; few differ from the oracle's own rounding
        au = O.verify_batch(om, [dict(req, K_stored=synth.as_f64(Kn), V_stored=synth.as_f64(Vn))])[0]["audit"]
        print(f"{kind}: {au['flips']} of {au['elements']} stored numbers differ from the oracle's rounding, "
              f"worst {au['max_excess']:.2e} of the vector's rms beyond a correct rounding")
        assert au["max_excess"] < 1e-4 and au["flips"] < 0.02 * au["elements"] and au["elements"] == 2 * Kn.numel()
    with pytest.raises(sled.SledError):
        v.read_kv(r, 30, 10)                 # past the request's pages
    v.destroy()
