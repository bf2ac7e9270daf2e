"""The serving loop on the GPU: queue, static batches, rounds, lost answers, sessions that end and start.
Whatever the drafters send and however the requests are batched, every device must end up with the
oracle's plain greedy continuation of its prompt (Sec. 3.1: verification is lossless; Sec. 3.2-3.4)."""
import numpy as np
import pytest
import torch

from oracle import sled_oracle as O
from paper_2506_09397_amd import serving, sled, synth
from gpu_common import build_verifier
from helpers import oracle_model

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind", ["tiny", "tiny_bf16"])
def test_serving_loop_is_lossless_under_batching_retries_and_churn(kind):
    shape = synth.SHAPES[kind]
    n_dev, n_new, batch = 6, 20, 4
    # a small pool: the second wave of sessions lives on pages that the first wave gave back
    v, w = build_verifier(shape, 7, n_pages=6 * 5 + 6, max_requests=n_dev, B_max=n_dev, ctx_tokens_max=n_dev * 96,
                          gain_jitter=0.1, std=0.08)
    om = oracle_model(shape, w)
    server = serving.Server(v, batch)
    lens = [5, 33, 17, 40, 9, 26, 12, 31, 3]
    prompts = [synth.context_tokens(L, shape.vocab, seed=70 + i).tolist() for i, L in enumerate(lens)]
    truth = [O.decode_greedy(om, p, n_new) for p in prompts]

    def run(devs, beta, lose_every, seed):
        drafters = {d: serving.ReplayDrafter(truth[d], shape.vocab, beta, seed=seed + d) for d in devs}
        first = {d: prompts[d][-1] for d in devs}
        return serving.simulate(server, drafters, first, n_new, k=5, draft_ms_per_token=1.0, seed=seed, lose_every=lose_every)

    wave1 = list(range(6))
    for d in wave1:
        server.open(d, prompt=prompts[d][:-1])
    res = run(wave1, beta=0.7, lose_every=4, seed=3)
    for d in wave1:
        assert res["texts"][d] == truth[d], f"device {d}"
    assert 0.2 < res["accepted_per_draft"] < 0.9
    assert res["steps"] < 6 * n_new            # speculation saved steps over one token per device and step
    # three sessions end, three new devices arrive and reuse their pages; the others keep generating nothing new
    for d in (0, 2, 4):
        server.close(d)
    wave2 = [6, 7, 8]
    for d in wave2:
        server.open(d, prompt=prompts[d][:-1])
    res2 = run(wave2, beta=0.4, lose_every=0, seed=5)
    for d in wave2:
        assert res2["texts"][d] == truth[d], f"device {d}"
    # a round that was answered cannot be asked for again with an older number
    with pytest.raises(ValueError):
        server.submit(6, 0, 1, [2])
    for d in (1, 3, 5, 6, 7, 8):
        server.close(d)
    # every page is back: six fresh sessions of 80 tokens fit again
    for d in range(6):
        server.open(d)
        K, V = synth.context_kv(shape, 80, seed=1, req=d, device="cuda")
        server.v.append_context([server.req_of[d]], [K], [V])
    assert server.v.lengths([server.req_of[d] for d in range(6)]) == [80] * 6
    v.destroy()


def test_static_batcher_order_and_duplicates():
    shape = synth.SHAPES["tiny"]
    v, w = build_verifier(shape, 2, n_pages=32, max_requests=4, B_max=4, ctx_tokens_max=256)
    server = serving.Server(v, 2)
    for d in range(3):
        server.open(d)
    assert server.run_batch() == []
    server.submit(0, 0, 5, [1, 2])
    assert not server.ready() and server.run_batch() == []
    server.submit(0, 1, 6, [])          # a second request of the same device must wait for the next step
    server.submit(1, 0, 7, [3])
    server.submit(2, 0, 8, [])
    r = server.run_batch()
    assert [(x.device, x.round_no) for x in r] == [(0, 0), (1, 0)]
    assert [p.device for p in server.queue] == [0, 2]
    r = server.run_batch()
    assert [(x.device, x.round_no) for x in r] == [(0, 1), (2, 0)]
    again = server.submit(1, 0, 7, [3, 4])
    assert again.replayed and again.round_no == 0
    v.destroy()
