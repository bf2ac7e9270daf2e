"""GPU parity of sled_verify_batch / sled_kv_append (+ sled_accept chained on their logits) against
the oracle, through the C ABI, on small models that still span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

from oracle import sled_oracle as O
from paper_2506_09397_amd import sled, synth
from gpu_common import build_verifier, oracle_requests
from helpers import oracle_model

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4      # max-abs logits error, fp32 models
TOL_BF16 = 2e-2     # max-abs logits error, bf16 models


def _dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).cuda()


def _setup_tiny_f32(seed=0, gain_jitter=0.0, std=0.02):
    shape = synth.SHAPES["tiny"]
    batch = synth.draw_batch("tiny4", shape.vocab, seed=seed)
    v, w = build_verifier(shape, seed, n_pages=96, max_requests=8, B_max=8, ctx_tokens_max=8 * 160,
                          gain_jitter=gain_jitter, std=std)
    om = oracle_model(shape, w)
    return shape, batch, v, w, om


def _oracle_chain(om, reqs_in, batch, mode, q=None, u_acc=None, u_smp=None):
    res = O.verify_batch(om, reqs_in)
    logits = np.concatenate([r["logits"] for r in res], axis=0)
    # the library returns float32 logits: the acceptance step sees those values
    logits32 = logits.astype(np.float32).astype(np.float64)
    acc = O.accept_batch(mode, batch.k, logits32, batch.tokens, q, u_acc, u_smp)
    return res, logits, acc


def test_tiny_fp32_step_greedy_and_sampling():
    """4 requests x 64 context tokens x 4 drafts on the 2-layer fp32 decoder, seed 0."""
    shape, batch, v, w, om = _setup_tiny_f32(0)
    reqs, Ks, Vs = [], [], []
    for i in range(batch.B):
        pf = O.prefill(om, synth.context_tokens(batch.ctx_len[i], shape.vocab, seed=i))
        reqs.append(v.open())
        Ks.append(_dev(pf["K"], torch.float32))
        Vs.append(_dev(pf["V"], torch.float32))
    v.append_context(reqs, Ks, Vs)
    assert v.lengths(reqs) == batch.ctx_len
    tokens = torch.from_numpy(batch.tokens).cuda()
    logits = v.verify(reqs, batch.k, tokens)
    torch.cuda.synchronize()
    got = logits.cpu().numpy().astype(np.float64)

    nd = sum(batch.k)
    q = synth.draft_probs(nd, shape.vocab, 0.5, seed=0, device="cuda")
    u_acc = synth.uniforms(nd, seed=1, device="cuda")
    u_smp = synth.uniforms(batch.B, seed=2, device="cuda")
    oreqs = oracle_requests(batch, Ks, Vs)
    res, want, acc_g = _oracle_chain(om, oreqs, batch, "greedy")
    err = np.abs(got - want).max()
    print(f"tiny fp32: max |logit error| = {err:.3e}")
    assert err < TOL_F32

    a, t = v.accept(sled.GREEDY, batch.k, logits, tokens)
    a, t = a.cpu().numpy(), t.cpu().numpy()
    for i, r in enumerate(acc_g):
        if r["margin"] > 10 * TOL_F32:
            assert (a[i], t[i]) == (r["accept_len"], r["out_token"])
    _, _, acc_s = _oracle_chain(om, oreqs, batch, "sample", synth.as_f64(q), synth.as_f64(u_acc), synth.as_f64(u_smp))
    a, t = v.accept(sled.SAMPLE, batch.k, logits, tokens, q, u_acc, u_smp)
    a, t = a.cpu().numpy(), t.cpu().numpy()
    n_checked = 0
    for i, r in enumerate(acc_s):
        if r["margin_acc"] > 100 * TOL_F32 and r["margin_cdf"] > 100 * TOL_F32 / shape.vocab * 10:
            assert (a[i], t[i]) == (r["accept_len"], r["out_token"])
            n_checked += 1
    assert n_checked >= 2

    # staged K/V of the new tokens: commit everything and read the lengths back
    v.commit(reqs, torch.tensor(batch.k, dtype=torch.int32, device="cuda"))
    assert v.lengths(reqs) == [L + k + 1 for L, k in zip(batch.ctx_len, batch.k)]
    v.destroy()


def test_tiny_fp32_gpu_prefill_by_chunked_verify_then_verify():
    """Context built on the GPU itself: chunks of k_max+1 tokens verified and fully committed
    (sled_kv_append with a device accept_len), then a ragged verify on top; also retry safety."""
    shape, _, v, w, om = _setup_tiny_f32(3, gain_jitter=0.1, std=0.05)
    ctx_len = [37, 64, 5, 16]
    k = [3, 0, 8, 4]
    batch = synth.make_batch(ctx_len, k, shape.vocab, seed=9)
    reqs = [v.open() for _ in ctx_len]
    ctx = [synth.context_tokens(L, shape.vocab, seed=20 + i) for i, L in enumerate(ctx_len)]
    step = shape.k_max + 1
    pos = 0
    while pos < max(ctx_len):
        rs, ks, toks = [], [], []
        for i, L in enumerate(ctx_len):
            n = min(step, L - pos)
            if n > 0:
                rs.append(reqs[i]); ks.append(n - 1); toks.append(ctx[i][pos: pos + n])
        tk = torch.from_numpy(np.concatenate(toks)).cuda()
        v.verify(rs, ks, tk)
        v.commit(rs, torch.tensor(ks, dtype=torch.int32, device="cuda"))
        pos += step
    assert v.lengths(reqs) == ctx_len
    tokens = torch.from_numpy(batch.tokens).cuda()
    first = v.verify(reqs, k, tokens).clone()
    again = v.verify(reqs, k, tokens).clone()        # never committed: issuing it again changes nothing
    torch.cuda.synchronize()
    assert torch.equal(first, again)
    oreqs = []
    offs = batch.row_offsets()
    for i in range(len(k)):
        pf = O.prefill(om, ctx[i])
        oreqs.append({"tokens": batch.tokens[offs[i]: offs[i + 1]], "K": pf["K"], "V": pf["V"]})
    want = np.concatenate([r["logits"] for r in O.verify_batch(om, oreqs)], axis=0)
    err = np.abs(first.cpu().numpy() - want).max()
    print(f"tiny fp32 (GPU-built context): max |logit error| = {err:.3e}")
    assert err < TOL_F32
    v.destroy()


BF16_CASES = [
    # ctx_len, k   (contexts off the page size, shorter than a page, empty; k from 0 to k_max)
    ([64, 64, 64, 64], [4, 4, 4, 4]),
    ([0, 5, 16, 17, 130, 257, 1000], [8, 0, 3, 8, 1, 7, 8]),
    ([300] * 20, [2, 4, 6, 8] * 5),           # 120 packed rows: one full row block of the projections
    ([200, 40, 333] * 15, [8, 7, 8] * 15),    # 405 packed rows: four row blocks sharing each weight tile, the last one ragged
    ([90] * 15, [8] * 15),                    # 135 packed rows: two row blocks, the second holding a single 32-row tile
]


@pytest.mark.parametrize("ctx_len,k", BF16_CASES)
def test_tiny_bf16_step(ctx_len, k):
    shape = synth.SHAPES["tiny_bf16"]
    B = len(k)
    v, w = build_verifier(shape, 1, n_pages=sum(ctx_len) // 16 + 3 * B + 8, max_requests=B, B_max=B,
                          ctx_tokens_max=sum(ctx_len) + 9 * B, gain_jitter=0.1, std=0.02)
    batch = synth.make_batch(ctx_len, k, shape.vocab, seed=4)
    reqs = [v.open() for _ in range(B)]
    Ks, Vs = [], []
    for i in range(B):
        K, V = synth.context_kv(shape, ctx_len[i], seed=2, req=i, device="cuda")
        Ks.append(K); Vs.append(V)
    v.append_context(reqs, Ks, Vs)
    tokens = torch.from_numpy(batch.tokens).cuda()
    got = v.verify(reqs, k, tokens).cpu().numpy().astype(np.float64)
    oreqs = oracle_requests(batch, Ks, Vs)
    want = np.concatenate([r["logits"] for r in O.verify_batch(oracle_model(shape, w), oreqs)], axis=0)
    exact = np.concatenate([r["logits"] for r in O.verify_batch(oracle_model(shape, w, "exact"), oreqs)], axis=0)
    err, err_exact = np.abs(got - want).max(), np.abs(got - exact).max()
    row_err = np.abs(got - want).max(axis=1)
    print(f"tiny bf16 B={B} T={batch.T}: max |logit error| = {err:.3e} (median row {np.median(row_err):.1e}; "
          f"vs unrounded oracle {err_exact:.3e}), logit std {want.std():.3f}")
    # Against the oracle with the same storage contract rows agree to about 1e-5 (bf16 pairs carry 16
    # bits), except where a new K/V value fell on the other side of a bf16 rounding boundary.
    assert err < TOL_BF16 / 4
    assert np.median(row_err) < 1e-3
    assert err_exact < TOL_BF16

    # a request's logits do not depend on its neighbours: verify request 1 alone
    if B > 2:
        i = 2
        offs = batch.row_offsets()
        alone = v.verify([reqs[i]], [k[i]], tokens[offs[i]: offs[i + 1]].contiguous()).cpu().numpy()
        assert np.abs(alone - got[offs[i]: offs[i + 1]]).max() < 2e-3
    v.destroy()


def test_bf16_results_do_not_depend_on_page_numbers():
    shape = synth.SHAPES["tiny_bf16"]
    ctx_len, k = [50, 33, 90], [3, 8, 5]
    batch = synth.make_batch(ctx_len, k, shape.vocab, seed=6)
    tokens = torch.from_numpy(batch.tokens).cuda()
    v, w = build_verifier(shape, 2, n_pages=64, max_requests=8, B_max=4, ctx_tokens_max=400)
    KV = [synth.context_kv(shape, L, seed=3, req=i, device="cuda") for i, L in enumerate(ctx_len)]

    def run(order, junk_first):
        junk = []
        if junk_first:       # occupy the first pages so the requests land elsewhere, then free them
            junk = [v.open() for _ in range(2)]
            jk = synth.context_kv(shape, 40, seed=9, req=99, device="cuda")
            v.append_context(junk, [jk[0]] * 2, [jk[1]] * 2)
        reqs = [None] * 3
        for i in order:
            reqs[i] = v.open()
            v.append_context([reqs[i]], [KV[i][0]], [KV[i][1]])
        for j in junk:
            v.close_request(j)
        out = v.verify(reqs, k, tokens).clone()
        torch.cuda.synchronize()
        for r in reqs:
            v.close_request(r)
        return out

    a = run([0, 1, 2], False)
    b = run([2, 0, 1], True)
    assert torch.equal(a, b)
    v.destroy()


def test_verify_argument_errors():
    shape = synth.SHAPES["tiny"]
    v, w = build_verifier(shape, 0, n_pages=4, max_requests=2, B_max=2, ctx_tokens_max=64)
    r0, r1 = v.open(), v.open()
    with pytest.raises(sled.SledError) as e:
        v.open()
    assert e.value.code == sled.ENOMEM
    tokens = torch.zeros(18, dtype=torch.int32, device="cuda")
    with pytest.raises(sled.SledError) as e:
        v.verify([r0], [9], tokens)                       # k above k_max
    assert e.value.code == sled.EINVAL
    with pytest.raises(sled.SledError) as e:
        v.verify([r0, r0], [1, 1], tokens)                # duplicate request
    assert e.value.code == sled.EINVAL
    with pytest.raises(sled.SledError) as e:
        v.commit([r0], torch.zeros(1, dtype=torch.int32, device="cuda"))   # nothing staged
    assert e.value.code == sled.ESTATE
    K, V = synth.context_kv(shape, 70, seed=1, req=0, device="cuda")
    with pytest.raises(sled.SledError) as e:
        v.append_context([r0], [K], [V])                  # 70 tokens need 5 pages, the pool has 4
    assert e.value.code == sled.ENOMEM
    v.destroy()


@pytest.mark.parametrize("kind", ["tiny", "tiny_bf16"])
def test_gpu_greedy_loop_reproduces_autoregressive_decoding(kind):
    """Several requests run the draft -> verify -> accept -> commit loop on the GPU (sled_verify_batch,
    sled_accept greedy, sled_kv_append with the device accept_len) with drafts that are partly right
    and partly wrong; the generated text must equal the oracle's plain one-token-at-a-time greedy
    decoding of the same prompts, token for token (Sec. 3.1: verification leaves the target's output
    unchanged)."""
    shape = synth.SHAPES[kind]
    B, n_new = 3, 24
    v, w = build_verifier(shape, 5, n_pages=64, max_requests=B, B_max=B, ctx_tokens_max=B * 96, gain_jitter=0.1,
                          std=0.08)
    om = oracle_model(shape, w)
    rng = np.random.default_rng(11)
    prompts = [synth.context_tokens(L, shape.vocab, seed=40 + i).tolist() for i, L in enumerate([9, 17, 3])]
    want = [O.decode_greedy(om, p, n_new) for p in prompts]

    reqs = [v.open() for _ in range(B)]
    # prompt ingestion through the same path: all prompt tokens but the last, in chunks, fully committed
    for i, p in enumerate(prompts):
        body = p[:-1]
        for s in range(0, len(body), shape.k_max + 1):
            chunk = body[s: s + shape.k_max + 1]
            tk = torch.tensor(chunk, dtype=torch.int32, device="cuda")
            v.verify([reqs[i]], [len(chunk) - 1], tk)
            v.commit([reqs[i]], torch.tensor([len(chunk) - 1], dtype=torch.int32, device="cuda"))
    pending = [p[-1] for p in prompts]
    out = [[] for _ in range(B)]
    rounds = 0
    while min(len(o) for o in out) < n_new:
        rounds += 1
        k, toks = [], []
        for i in range(B):
            # drafts: the true continuation, corrupted from a random position on; random length 0..k_max
            ki = int(rng.integers(0, shape.k_max + 1))
            truth = want[i][len(out[i]): len(out[i]) + ki]
            drafts = list(truth) + [int(x) for x in rng.integers(0, shape.vocab, size=ki - len(truth))]
            cut = int(rng.integers(0, ki + 1))
            drafts[cut:] = [int(x) for x in rng.integers(0, shape.vocab, size=ki - cut)]
            k.append(ki)
            toks += [pending[i]] + drafts
        tokens = torch.tensor(toks, dtype=torch.int32, device="cuda")
        logits = v.verify(reqs, k, tokens)
        a, t = v.accept(sled.GREEDY, k, logits, tokens)
        v.commit(reqs, a)
        a, t = a.cpu().numpy(), t.cpu().numpy()
        row = 0
        for i in range(B):
            drafts = toks[row + 1: row + 1 + k[i]]
            out[i] += drafts[: a[i]] + [int(t[i])]
            pending[i] = int(t[i])
            row += k[i] + 1
    for i in range(B):
        assert out[i][:n_new] == want[i], f"request {i} diverged after {rounds} rounds"
    # the cache holds the prompt body, every emitted token but the pending one
    assert v.lengths(reqs) == [len(p) - 1 + len(o) for p, o in zip(prompts, out)]
    v.destroy()
