"""GPU parity at the other benchmark shapes, at reduced depth (every layer shape, two layers):

  * the heterogeneous 64-request mix (contexts log-uniform in [128, 8192], k in {2,4,6,8}) on the
    Llama-3-8B shape with speculative-sampling acceptance over full-vocabulary draft probabilities;
  * the 70B shape (d 8192, 64/8 heads: 8 query heads per kv head, so up to 72 stacked query rows per
    attention tile) with 32 requests, contexts uniform in [1024, 4096], k uniform in [4, 8].

The oracle scores a sample of the requests (requests are independent); acceptance is compared on the
logits the library produced, so that its decisions are judged on identical inputs.
"""
import time

import numpy as np
import pytest
import torch

from oracle import sled_oracle as O
from paper_2506_09397_amd import sled, synth
from gpu_common import build_verifier, MARGIN_ACC, MARGIN_CDF
from helpers import oracle_model

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


def _setup(shape, batch, seed, keep):
    B = batch.B
    ctx_budget = sum(batch.ctx_len) + 9 * B
    v, w = build_verifier(shape, seed, n_pages=ctx_budget // 16 + 2 * B + 8, max_requests=B, B_max=B,
                          ctx_tokens_max=ctx_budget)
    reqs, KV = [], {}
    for i in range(B):
        K, V = synth.context_kv(shape, batch.ctx_len[i], seed=seed, req=i, device="cuda")
        reqs.append(v.open())
        v.append_context([reqs[i]], [K], [V])
        if i in keep:
            KV[i] = (K.cpu(), V.cpu())
    return v, w, reqs, KV


def _sample_requests(batch, n):
    """Longest, shortest and a spread of the others."""
    order = np.argsort(batch.ctx_len)
    pick = {int(order[0]), int(order[-1])}
    for j in np.linspace(0, batch.B - 1, n).astype(int):
        pick.add(int(order[j]))
    return sorted(pick)[: max(n, 2)]


def _logit_errors(shape, w, batch, KV, got, sample, label):
    offs = batch.row_offsets()
    oreqs = [{"tokens": batch.tokens[offs[i]: offs[i + 1]], "K": synth.as_f64(KV[i][0]), "V": synth.as_f64(KV[i][1])}
             for i in sample]
    t0 = time.time()
    res = O.verify_batch(oracle_model(shape, w), oreqs)
    dt = time.time() - t0
    errs = []
    for i, r in zip(sample, res):
        e = float(np.abs(got[offs[i]: offs[i + 1]] - r["logits"]).max())
        errs.append(e)
        print(f"{label}: request {i} (L={batch.ctx_len[i]}, k={batch.k[i]}): max |logit error| {e:.3e}")
    print(f"{label}: oracle time for {len(sample)} requests {dt:.1f} s")
    return errs


def test_llama8b_hetero64_sampling_two_layers():
    shape = synth.scaled_shape(synth.SHAPES["llama8b"], n_layers=2)
    batch = synth.draw_batch("hetero64", shape.vocab, seed=0)
    sample = _sample_requests(batch, 6)
    v, w, reqs, KV = _setup(shape, batch, 0, set(sample))
    tokens = torch.from_numpy(batch.tokens).cuda()
    logits = v.verify(reqs, batch.k, tokens)
    got = logits.cpu().numpy()
    assert np.isfinite(got).all()
    errs = _logit_errors(shape, w, batch, KV, got, sample, f"8B shape, hetero64 (T={batch.T})")
    assert max(errs) < TOL_BF16

    # speculative sampling over full-vocabulary draft probabilities, on the library's own logits
    nd = int(sum(batch.k))
    q = synth.draft_probs(nd, shape.vocab, 1.0, seed=3, device="cuda", base_std=1.28)
    u_acc = synth.uniforms(nd, seed=4, device="cuda")
    u_smp = synth.uniforms(batch.B, seed=5, device="cuda")
    a, t = v.accept(sled.SAMPLE, batch.k, logits, tokens, q, u_acc, u_smp)
    a, t = a.cpu().numpy(), t.cpu().numpy()
    want = O.accept_batch("sample", batch.k, got.astype(np.float64), batch.tokens, synth.as_f64(q),
                          synth.as_f64(u_acc), synth.as_f64(u_smp))
    n_sub = 0
    for i, r in enumerate(want):
        if r["margin_acc"] > MARGIN_ACC and r["margin_cdf"] > MARGIN_CDF:
            assert (int(a[i]), int(t[i])) == (r["accept_len"], r["out_token"]), f"request {i}"
        else:
            n_sub += 1
            assert 0 <= a[i] <= batch.k[i]
    print(f"sampling acceptance: {batch.B - n_sub} of {batch.B} requests compared exactly, "
          f"mean accepted {np.mean(a):.2f} of mean k {np.mean(batch.k):.2f}")
    assert n_sub <= 2
    # commit and check the lengths moved by accept_len + 1
    v.commit(reqs, v.accept_len[: batch.B])
    assert v.lengths(reqs) == [L + int(x) + 1 for L, x in zip(batch.ctx_len, a)]
    v.destroy()


def test_llama70b_shape_two_layers():
    shape = synth.scaled_shape(synth.SHAPES["llama70b"], n_layers=2)
    batch = synth.draw_batch("b32", shape.vocab, seed=0)
    sample = _sample_requests(batch, 3)
    v, w, reqs, KV = _setup(shape, batch, 0, set(sample))
    tokens = torch.from_numpy(batch.tokens).cuda()
    logits = v.verify(reqs, batch.k, tokens)
    got = logits.cpu().numpy()
    assert np.isfinite(got).all()
    errs = _logit_errors(shape, w, batch, KV, got, sample, f"70B shape, b32 (T={batch.T})")
    assert max(errs) < TOL_BF16
    a, t = v.accept(sled.GREEDY, batch.k, logits, tokens)
    want = O.accept_batch("greedy", batch.k, got.astype(np.float64), batch.tokens)
    a, t = a.cpu().numpy(), t.cpu().numpy()
    for i, r in enumerate(want):
        if r["margin"] > 0:
            assert (int(a[i]), int(t[i])) == (r["accept_len"], r["out_token"]), f"request {i}"
    v.destroy()


def test_512_rows_four_row_blocks_per_weight_tile():
    """512 packed rows on the 8B layer shape (one layer, vocabulary 65536): every projection runs in the wide
    workgroup shape with four 128-row blocks per weight tile (split-K partials, SwiGLU and logits epilogues).
    All rows of a sample of requests against the oracle."""
    shape = synth.scaled_shape(synth.SHAPES["llama8b"], n_layers=1, vocab=65536)
    B = 64
    batch = synth.make_batch([16 + (i % 5) for i in range(B)], [7] * B, shape.vocab, seed=21)
    assert batch.T == 512
    sample = [0, 9, 17, 31, 32, 47, 63]    # rows from all four blocks
    v, w, reqs, KV = _setup(shape, batch, 6, set(sample))
    got = v.verify(reqs, batch.k, torch.from_numpy(batch.tokens).cuda()).cpu().numpy().astype(np.float64)
    errs = _logit_errors(shape, w, batch, KV, got, sample, "8B layer shape, 512 rows")
    assert max(errs) < TOL_BF16
    v.destroy()


@pytest.mark.parametrize("n_q,n_kv,k_max,ks", [
    (8, 2, 8, [3, 0, 2, 1, 3]),           # G = 4, at most 16 query rows per (request, kv head): one query tile
    (8, 2, 8, [7, 4, 5, 0]),              # 32 rows: two tiles
    (8, 2, 15, [15, 12, 0, 7, 13, 15]),   # 64 rows: four tiles, drafts of up to 15 tokens
    (8, 1, 9, [9, 4, 8, 0]),              # G = 8, 80 rows: five tiles, the largest supported
    (8, 8, 15, [15, 3, 9]),               # no grouping (G = 1) with the longest drafts
])
def test_every_query_tile_count_of_the_attention_kernel(n_q, n_kv, k_max, ks):
    """The attention kernel is instantiated for one to five 16-row query tiles per (request, kv head), chosen from
    the batch's longest draft and the model's group size; every instantiation against the oracle, with contexts that
    end inside a page, are shorter than a page, or are empty."""
    from oracle import sled_oracle as O
    from paper_2506_09397_amd.runtime import Verifier
    from helpers import oracle_model, oracle_requests
    shape = synth.scaled_shape(synth.SHAPES["tiny_bf16"], n_q_heads=n_q, n_kv_heads=n_kv, k_max=k_max)
    w = synth.SynthWeights(shape, seed=9, device="cuda", std=0.03, gain_jitter=0.1)
    B = len(ks)
    ctx_len = [0, 5, 16, 131, 700, 257][:B]
    budget = sum(ctx_len) + (k_max + 1) * B
    v = Verifier(shape, w, budget // 16 + 3 * B + 8, B, B, budget)
    batch = synth.make_batch(ctx_len, ks, shape.vocab, seed=3)
    reqs = [v.open() for _ in range(B)]
    Ks, Vs = [], []
    for i in range(B):
        K, V = synth.context_kv(shape, ctx_len[i], seed=3, req=i, device="cuda")
        Ks.append(K); Vs.append(V)
    v.append_context(reqs, Ks, Vs)
    got = v.verify(reqs, ks, torch.from_numpy(batch.tokens).cuda()).cpu().numpy().astype(np.float64)
    want = np.concatenate([r["logits"] for r in O.verify_batch(oracle_model(shape, w), oracle_requests(batch, Ks, Vs))], axis=0)
    err = np.abs(got - want).max()
    print(f"Hq/Hkv={n_q}/{n_kv} k_max={k_max} k={ks}: max |logit error| = {err:.3e} (logit std {want.std():.3f})")
    assert err < 5e-3
    v.destroy()
