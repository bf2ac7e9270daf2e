"""Pins for the oracle's acceptance step (CPU only).

Checked against what Eq. 1 (Sec. 3.1) and the paper's losslessness statement fix:
  * hand-derived rational examples (tests/golden/eq1_worked_examples.txt);
  * exact enumeration over a grid of uniforms with rational arithmetic;
  * the emitted tokens follow the target distribution exactly (chi-square over many
    seeded trials) and the per-token acceptance rate is sum_v min(p, q);
  * invariants: accepted length within [0, k]; identical distributions accept everything;
    a rejected draft is never re-emitted; greedy verification of the target's own argmax
    chain accepts everything; ties go to the lowest token id;
  * the draft -> verify -> commit loop with greedy verification reproduces plain
    autoregressive greedy decoding token for token on a tiny model.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

from oracle import sled_oracle as O
from paper_2506_09397_amd import synth
from helpers import oracle_model

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "eq1_worked_examples.txt")


def _golden_cases():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, p, q, alpha, resid, beta = [f.strip() for f in line.split("|")]
        fr = lambda s: [Fraction(x) for x in s.split()]
        cases.append((name, fr(p), fr(q), fr(alpha), None if "-" in resid else fr(resid), Fraction(beta)))
    return cases


@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: c[0])
def test_golden_eq1_examples(case):
    name, p, q, alpha, resid, beta = case
    V = len(p)
    logits = np.log(np.array([[float(x) for x in p]] * 2))
    qa = np.array([[float(x) for x in q]])
    eps = 1e-9
    for d in range(V):
        a = float(alpha[d])
        if a < 1:
            # just under alpha: accepted; just over: rejected
            assert O.accept_sample(logits, [d], qa, [a - eps], 0.5)["accept_len"] == 1
            rej = O.accept_sample(logits, [d], qa, [a + eps], 0.5)
            assert rej["accept_len"] == 0
            # resample: inverse CDF of the residual, scanned in ascending token order
            cdf = np.cumsum([float(x) for x in resid])
            for u in np.linspace(0.003, 0.997, 41):
                want = int(np.nonzero(cdf > u)[0][0])
                got = O.accept_sample(logits, [d], qa, [a + eps], float(u))["out_token"]
                assert got == want
        else:
            assert O.accept_sample(logits, [d], qa, [1.0 - eps], 0.5)["accept_len"] == 1
    assert sum(min(a, b) for a, b in zip(p, q)) == beta


def test_exhaustive_grid_against_rational_enumeration():
    """k = 2, V = 4: enumerate the outcome on a grid of (u1, u2, u') with exact fractions."""
    P = [[Fraction(1, 8), Fraction(3, 8), Fraction(1, 4), Fraction(1, 4)],
         [Fraction(2, 5), Fraction(1, 10), Fraction(1, 5), Fraction(3, 10)],
         [Fraction(1, 10), Fraction(1, 5), Fraction(3, 10), Fraction(2, 5)]]
    Q = [[Fraction(1, 4), Fraction(1, 4), Fraction(1, 4), Fraction(1, 4)],
         [Fraction(1, 10), Fraction(2, 5), Fraction(2, 5), Fraction(1, 10)]]
    logits = np.log(np.array([[float(x) for x in r] for r in P]))
    q = np.array([[float(x) for x in r] for r in Q])
    grid = [Fraction(2 * i + 1, 34) for i in range(17)]       # never on a boundary of these fractions

    def draw(w, u):
        tot, c = sum(w), Fraction(0)
        for v, x in enumerate(w):
            c += x
            if c > u * tot:
                return v
        raise AssertionError

    n = 0
    for d1 in range(4):
        for d2 in range(4):
            for u1 in grid:
                for u2 in grid[::4]:
                    for us in grid[::2]:
                        if u1 * Q[0][d1] > P[0][d1]:
                            want = (0, draw([max(Fraction(0), a - b) for a, b in zip(P[0], Q[0])], us))
                        elif u2 * Q[1][d2] > P[1][d2]:
                            want = (1, draw([max(Fraction(0), a - b) for a, b in zip(P[1], Q[1])], us))
                        else:
                            want = (2, draw(P[2], us))
                        r = O.accept_sample(logits, [d1, d2], q, [float(u1), float(u2)], float(us))
                        assert (r["accept_len"], r["out_token"]) == want
                        n += 1
    assert n > 5000


def _random_dists(rng, rows, V, sharp=1.5):
    z = rng.standard_normal((rows, V)) * sharp
    e = np.exp(z - z.max(axis=1, keepdims=True))
    return z, e / e.sum(axis=1, keepdims=True)


def test_sampling_preserves_target_distribution_chi_square():
    """Losslessness (Sec. 3.1): the first emitted token follows p_0 and, given the first draft
    was accepted, the second follows p_1; acceptance rate of draft 1 is sum min(p, q)."""
    rng = np.random.default_rng(1234)
    V, k, N = 12, 3, 30000
    z, p = _random_dists(rng, k + 1, V)
    _, q = _random_dists(rng, k, V)
    first = np.zeros(V)
    second = np.zeros(V)
    n_acc1 = 0
    for _ in range(N):
        drafts = [int(rng.choice(V, p=q[j])) for j in range(k)]
        r = O.accept_sample(z, drafts, q, rng.random(k), rng.random())
        emitted = drafts[: r["accept_len"]] + [r["out_token"]]
        first[emitted[0]] += 1
        if r["accept_len"] >= 1:
            n_acc1 += 1
            second[emitted[1]] += 1
    assert stats.chisquare(first, p[0] * N).pvalue > 1e-3
    assert stats.chisquare(second, p[1] * second.sum()).pvalue > 1e-3
    beta = np.minimum(p[0], q[0]).sum()
    assert abs(n_acc1 / N - beta) < 4 * math.sqrt(beta * (1 - beta) / N)
    # a wrong residual (e.g. resampling from p instead of max(0, p-q)) must fail this test
    wrong = np.zeros(V)
    rng2 = np.random.default_rng(99)
    for _ in range(N):
        d = int(rng2.choice(V, p=q[0]))
        if rng2.random() * q[0][d] <= p[0][d]:
            wrong[d] += 1
        else:
            wrong[int(rng2.choice(V, p=p[0]))] += 1
    assert stats.chisquare(wrong, p[0] * N).pvalue < 1e-6


def test_truncated_draft_distribution_is_lossless_when_the_draft_was_drawn_from_it():
    """A device that drafts from its top-m tokens renormalised and sends only those m (id, probability) pairs
    loses nothing: Eq. 1 with that truncated q still emits exactly p.  Using the truncated q for a draft that
    was drawn from the FULL q, however, is not lossless -- so the exactness is a property of how the draft was
    drawn, which the sparse entry point's contract states."""
    rng = np.random.default_rng(77)
    V, m, N = 12, 4, 30000
    z, p = _random_dists(rng, 2, V)
    _, q_full = _random_dists(rng, 1, V, sharp=1.0)
    top = np.argsort(-q_full[0])[:m]
    q_trunc = np.zeros((1, V))
    q_trunc[0, top] = q_full[0, top] / q_full[0, top].sum()
    good = np.zeros(V)
    bad = np.zeros(V)
    for _ in range(N):
        d = int(rng.choice(V, p=q_trunc[0]))
        r = O.accept_sample(z, [d], q_trunc, rng.random(1), rng.random())
        good[([d][: r["accept_len"]] + [r["out_token"]])[0]] += 1
        d = int(rng.choice(V, p=q_full[0]))
        r = O.accept_sample(z, [d], q_trunc, rng.random(1), rng.random())
        bad[([d][: r["accept_len"]] + [r["out_token"]])[0]] += 1
    assert stats.chisquare(good, p[0] * N).pvalue > 1e-3
    assert stats.chisquare(bad, p[0] * N).pvalue < 1e-6


def test_top_m_plus_remainder_mass_is_lossless_when_the_draft_was_drawn_from_the_reconstruction():
    """The cheaper uplink with less distortion of the drafter: the device sends its top-m (id, probability) pairs as
    they are plus the mass rho of everything else, and both sides agree that rho is spread evenly over the tokens that
    are not listed.  Eq. 1 with that reconstructed distribution emits exactly p if the device drew its draft from the
    reconstruction (top-m as is, with probability rho a uniformly random unlisted token) -- and not if it drew from its
    full distribution, whose tail the server never saw.  Its acceptance rate beta = sum min(p, q) is at least that of
    the renormalised top-m whenever the target puts weight on the tail."""
    rng = np.random.default_rng(78)
    V, m, N = 12, 4, 30000
    z, p = _random_dists(rng, 2, V)
    _, q_full = _random_dists(rng, 1, V, sharp=1.0)
    top = np.argsort(-q_full[0])[:m]
    rho = 1.0 - q_full[0, top].sum()
    q_rec = np.full((1, V), rho / (V - m))
    q_rec[0, top] = q_full[0, top]
    assert abs(q_rec.sum() - 1.0) < 1e-12 and 0.05 < rho < 0.95
    good, bad = np.zeros(V), np.zeros(V)
    for _ in range(N):
        d = int(rng.choice(V, p=q_rec[0]))
        r = O.accept_sample(z, [d], q_rec, rng.random(1), rng.random())
        good[([d][: r["accept_len"]] + [r["out_token"]])[0]] += 1
        d = int(rng.choice(V, p=q_full[0]))
        r = O.accept_sample(z, [d], q_rec, rng.random(1), rng.random())
        bad[([d][: r["accept_len"]] + [r["out_token"]])[0]] += 1
    assert stats.chisquare(good, p[0] * N).pvalue > 1e-3
    assert stats.chisquare(bad, p[0] * N).pvalue < 1e-6
    q_ren = np.zeros(V)
    q_ren[top] = q_full[0, top] / q_full[0, top].sum()
    assert np.minimum(p[0], q_rec[0]).sum() > np.minimum(p[0], q_ren).sum()


def test_expected_accept_length_closed_form():
    """Same (p, q) in every row: E[accept_len] = beta (1 - beta^k) / (1 - beta)."""
    rng = np.random.default_rng(5)
    V, k, N = 16, 4, 20000
    z1, p1 = _random_dists(rng, 1, V)
    _, q1 = _random_dists(rng, 1, V)
    z = np.repeat(z1, k + 1, axis=0)
    q = np.repeat(q1, k, axis=0)
    beta = np.minimum(p1[0], q1[0]).sum()
    want = beta * (1 - beta ** k) / (1 - beta)
    tot = 0
    for _ in range(N):
        drafts = rng.choice(V, size=k, p=q1[0])
        tot += O.accept_sample(z, drafts, q, rng.random(k), rng.random())["accept_len"]
    assert abs(tot / N - want) < 0.05


def test_sampling_invariants():
    rng = np.random.default_rng(7)
    for trial in range(300):
        V = int(rng.integers(2, 40))
        k = int(rng.integers(0, 6))
        z, p = _random_dists(rng, k + 1, V)
        _, q = _random_dists(rng, max(k, 1), V)
        q = q[:k]
        drafts = rng.integers(0, V, size=k)
        r = O.accept_sample(z, drafts, q, rng.random(k), rng.random())
        a, t = r["accept_len"], r["out_token"]
        assert 0 <= a <= k and 0 <= t < V
        if a < k:  # rejected draft: it had p < q, so it has no residual mass and cannot come back
            assert t != drafts[a]
            assert p[a][t] - q[a][t] > 0
        # identical distributions: everything is accepted whatever the uniforms
        r2 = O.accept_sample(z, drafts, p[:k], rng.random(k), rng.random())
        assert r2["accept_len"] == k
    # one-hot draft distribution at d: accepted with probability p(d)
    z, p = _random_dists(rng, 2, 6)
    onehot = np.zeros((1, 6)); onehot[0, 2] = 1.0
    assert O.accept_sample(z, [2], onehot, [p[0][2] * 0.999], 0.3)["accept_len"] == 1
    assert O.accept_sample(z, [2], onehot, [min(p[0][2] * 1.001, 1.0)], 0.3)["accept_len"] == 0
    # q(d) = 0 can only be accepted (p/q is unbounded)
    q0 = np.full((1, 6), 0.2); q0[0, 4] = 0.0
    assert O.accept_sample(z, [4], q0, [0.9999], 0.3)["accept_len"] == 1


def test_draft_outside_the_vocabulary_is_rejected_where_it_stands():
    """A device may send any integer: an id outside [0, V) has no target probability, so the accepted prefix ends
    there, whatever the uniforms, and the corrective token comes from that position's residual (Eq. 1)."""
    rng = np.random.default_rng(21)
    z, p = _random_dists(rng, 4, 12)
    _, q = _random_dists(rng, 3, 12)
    good = [int(np.argmax(p[0])), int(np.argmax(p[1])), int(np.argmax(p[2]))]
    for bad in (-1, 12, 10**6, -(2**31)):
        for pos in range(3):
            drafts = list(good)
            drafts[pos] = bad
            r = O.accept_sample(z, drafts, q, [0.0] * 3, 0.37)     # u = 0 would accept every in-vocabulary draft
            assert r["accept_len"] == pos and 0 <= r["out_token"] < 12
            want, _ = O.inverse_cdf(np.maximum(0.0, p[pos] - q[pos]), 0.37)
            assert r["out_token"] == want
            g = O.accept_greedy(z, drafts)
            assert g["accept_len"] <= pos


def test_temperature_is_logit_scaling():
    rng = np.random.default_rng(8)
    z, _ = _random_dists(rng, 4, 10)
    _, q = _random_dists(rng, 3, 10)
    for _ in range(50):
        d = rng.integers(0, 10, size=3); ua = rng.random(3); us = rng.random()
        a = O.accept_sample(z, d, q, ua, us, temperature=2.0)
        b = O.accept_sample(z / 2.0, d, q, ua, us, temperature=1.0)
        assert (a["accept_len"], a["out_token"]) == (b["accept_len"], b["out_token"])


def test_inverse_cdf_cells():
    w = np.array([0.0, 2.0, 0.0, 1.0, 1.0, 0.0])
    assert O.inverse_cdf(w, 0.0)[0] == 1
    assert O.inverse_cdf(w, 0.49)[0] == 1
    assert O.inverse_cdf(w, 0.5)[0] == 3          # C(1) = 2 is not > 2
    assert O.inverse_cdf(w, 0.74)[0] == 3
    assert O.inverse_cdf(w, 0.76)[0] == 4
    assert O.inverse_cdf(w, 1.0)[0] == 4          # fallback: last index with mass
    v, margin = O.inverse_cdf(w, 0.6)
    assert v == 3 and abs(margin - 0.1) < 1e-15


def test_greedy_rules():
    z = np.array([[0.0, 3.0, 1.0], [5.0, 5.0, 1.0], [0.0, 1.0, 9.0], [2.0, 2.0, 2.0]])
    # argmax chain is [1, 0 (tie -> lowest id), 2, 0]
    assert O.accept_greedy(z, [1, 0, 2])["accept_len"] == 3
    assert O.accept_greedy(z, [1, 0, 2])["out_token"] == 0
    r = O.accept_greedy(z, [1, 1, 2])        # second draft hits the higher id of a tie: rejected
    assert (r["accept_len"], r["out_token"]) == (1, 0)
    r = O.accept_greedy(z, [2, 0, 2])
    assert (r["accept_len"], r["out_token"]) == (0, 1)
    r = O.accept_greedy(z[:1], [])           # k = 0: plain decode step
    assert (r["accept_len"], r["out_token"]) == (0, 1)
    assert O.accept_greedy(z, [1, 0, 2])["margin"] == 0.0   # the tie shows up as a zero margin


def test_accept_batch_packing():
    rng = np.random.default_rng(11)
    k = [2, 0, 3, 1]
    T, V = sum(k) + len(k), 9
    z, _ = _random_dists(rng, T, V)
    _, q = _random_dists(rng, sum(k), V)
    toks = rng.integers(0, V, size=T).astype(np.int32)
    ua, us = rng.random(sum(k)), rng.random(len(k))
    got = O.accept_batch("sample", k, z, toks, q, ua, us)
    row = dr = 0
    for i, ki in enumerate(k):
        want = O.accept_sample(z[row:row + ki + 1], toks[row + 1: row + 1 + ki], q[dr:dr + ki], ua[dr:dr + ki], us[i])
        assert (got[i]["accept_len"], got[i]["out_token"]) == (want["accept_len"], want["out_token"])
        row += ki + 1; dr += ki
    gg = O.accept_batch("greedy", k, z, toks)
    assert all(0 <= g["accept_len"] <= ki for g, ki in zip(gg, k))


TINY = synth.ModelShape(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=64,
                        vocab=48, dtype="f32", rope_theta=10000.0)


@pytest.mark.parametrize("drafter_kind", ["random", "corrupted_truth", "perfect", "empty"])
def test_greedy_verify_loop_equals_autoregressive_decoding(drafter_kind):
    """Sec. 3.1 / abstract: verification does not change what the target would have generated."""
    shape = TINY
    om = oracle_model(shape, synth.SynthWeights(shape, seed=21, std=0.3))
    prompt = synth.context_tokens(7, shape.vocab, seed=1).tolist()
    n_new = 14
    truth = O.decode_greedy(om, prompt, n_new + 8)
    rng = np.random.default_rng(3)

    def drafter(hist):
        done = len(hist) - len(prompt)
        kk = int(rng.integers(1, 6))
        if drafter_kind == "empty":
            return []
        if drafter_kind == "random":
            return rng.integers(0, shape.vocab, size=kk).tolist()
        guess = list(truth[done: done + kk])
        if drafter_kind == "corrupted_truth" and guess and rng.random() < 0.6:
            j = int(rng.integers(0, len(guess)))
            guess[j] = (guess[j] + 1) % shape.vocab
        return guess

    got, acc = O.speculative_greedy(om, prompt, n_new, drafter)
    assert got == truth[:n_new]
    if drafter_kind == "perfect":
        assert sum(acc) > 0 and len(acc) < n_new      # drafts were accepted: fewer rounds than tokens
    if drafter_kind == "empty":
        assert acc == [0] * n_new


def test_row_confidence_closed_forms():
    """Pins of the confidence score (Eq. 2): two classes give the logistic function of the logit gap over the
    temperature; equal logits give 1/V with the lowest id; a shift of all logits changes nothing; the
    temperature interpolates between 1/V and 1; and the score is the largest entry of a library softmax."""
    from scipy.special import softmax as scipy_softmax
    rng = np.random.default_rng(11)
    for a, b, tau in ((0.3, -1.2, 1.0), (2.0, 2.5, 0.7), (-4.0, 3.0, 2.0)):
        conf, top = O.row_confidence(np.array([[a, b]]), tau)
        assert top[0] == (0 if a >= b else 1)
        assert conf[0] == pytest.approx(1.0 / (1.0 + math.exp(-abs(a - b) / tau)), rel=1e-14)
    conf, top = O.row_confidence(np.full((3, 17), 0.25))
    assert np.allclose(conf, 1.0 / 17, rtol=1e-15) and (top == 0).all()
    z = rng.normal(0, 2, size=(5, 300))
    c0, t0 = O.row_confidence(z, 0.8)
    c1, t1 = O.row_confidence(z + 123.5, 0.8)
    assert np.allclose(c0, c1, rtol=1e-12) and (t0 == t1).all()
    lib = scipy_softmax(z / 0.8, axis=1)
    assert np.allclose(c0, lib.max(axis=1), rtol=1e-12) and (t0 == lib.argmax(axis=1)).all()
    hot, _ = O.row_confidence(z, 1e-3)
    cold, _ = O.row_confidence(z, 1e6)
    assert np.allclose(hot, 1.0, atol=1e-9) and np.allclose(cold, 1.0 / 300, rtol=1e-4)
    z[2, 40] = z[2, 7] = z[2].max() + 1.0          # a tie: the lower id wins, the score counts one of them
    c2, t2 = O.row_confidence(z)
    assert t2[2] == 7 and c2[2] == pytest.approx(lib_max_of(z[2]), rel=1e-12)


def lib_max_of(row):
    from scipy.special import softmax as scipy_softmax
    return scipy_softmax(row).max()
