"""Host logic of the serving loop (queue, static batches, replayed answers, the device simulation) against a
stand-in verifier that runs on the CPU: a toy 'target model' whose next token is a fixed function of the
context, with the same accept rule (greedy prefix match)."""
import numpy as np
import pytest
import torch

from paper_2506_09397_amd import serving, sled


class ToyShape:
    k_max = 8
    vocab = 97


class ToyVerifier:
    """Keeps each request's committed tokens; logits row j puts all mass on f(context + tokens[0..j])."""
    shape = ToyShape()

    def __init__(self):
        self.ctx = {}
        self.staged = {}
        self.next_id = 0
        self.calls = 0

    @staticmethod
    def f(seq):
        h = 7
        for t in seq:
            h = (h * 31 + int(t) + 1) % 1000003
        return h % ToyShape.vocab

    def open(self):
        self.next_id += 1
        self.ctx[self.next_id] = []
        return self.next_id

    def close_request(self, r):
        del self.ctx[r]

    def append_context(self, reqs, K, V):
        raise AssertionError("not used")

    def prefill(self, r, tokens, want_logits=True):
        self.ctx[r] += tokens.tolist()

    def verify(self, reqs, k, tokens):
        self.calls += 1
        toks = tokens.tolist()
        rows, off = [], 0
        for r, ki in zip(reqs, k):
            mine = toks[off: off + ki + 1]
            self.staged[r] = mine
            for j in range(ki + 1):
                row = torch.zeros(ToyShape.vocab)
                row[self.f(self.ctx[r] + mine[: j + 1])] = 1.0
                rows.append(row)
            off += ki + 1
        return torch.stack(rows)

    def accept(self, mode, k, logits, tokens):
        assert mode == sled.GREEDY
        toks = tokens.tolist()
        a, t, off = [], [], 0
        for ki in k:
            best = logits[off: off + ki + 1].argmax(dim=1).tolist()
            n = 0
            while n < ki and toks[off + 1 + n] == best[n]:
                n += 1
            a.append(n)
            t.append(best[n])
            off += ki + 1
        return torch.tensor(a, dtype=torch.int32), torch.tensor(t, dtype=torch.int32)

    def commit(self, reqs, a):
        for r, ai in zip(reqs, a.tolist()):
            self.ctx[r] += self.staged.pop(r)[: ai + 1]

    def lengths(self, reqs):
        return [len(self.ctx[r]) for r in reqs]


def toy_truth(start, n):
    seq, out = list(start), []
    for _ in range(n):
        out.append(ToyVerifier.f(seq))
        seq.append(out[-1])
    return out


def test_batches_are_fifo_one_request_per_device_and_answers_replay():
    v = ToyVerifier()
    s = serving.Server(v, 2, device="cpu")
    for d in range(3):
        s.open(d)
    assert s.run_batch() == [] and not s.ready()
    s.submit(0, 0, 5, [1, 2])
    s.submit(0, 1, 6, [])
    s.submit(1, 0, 7, [3])
    s.submit(2, 0, 8, [])
    r = s.run_batch()
    assert [(x.device, x.round_no) for x in r] == [(0, 0), (1, 0)]
    assert [p.device for p in s.queue] == [0, 2]
    calls = v.calls
    again = s.submit(1, 0, 7, [3, 4, 5])             # lost answer, sent again with more drafts
    assert again.replayed and (again.accept_len, again.out_token) == (r[1].accept_len, r[1].out_token)
    assert v.calls == calls and len(s.queue) == 2    # nothing verified twice, nothing queued
    r = s.run_batch()
    assert [(x.device, x.round_no) for x in r] == [(0, 1), (2, 0)]
    with pytest.raises(ValueError):
        s.submit(0, 0, 5, [1])
    long = list(range(20))
    s.submit(2, 1, r[1].out_token, long)
    assert len(s.queue[-1].drafts) == ToyShape.k_max  # longer drafts are cut to what one step can take
    s.close(2)
    assert all(p.device != 2 for p in s.queue)


@pytest.mark.parametrize("beta,lose_every,batch", [(1.0, 0, 4), (0.6, 3, 3), (0.0, 0, 1), (0.8, 2, 8)])
def test_simulation_ends_with_the_targets_own_text(beta, lose_every, batch):
    v = ToyVerifier()
    s = serving.Server(v, batch, device="cpu")
    n_dev, n_new, k = 5, 30, 4
    first = {d: 10 + d for d in range(n_dev)}
    truth = {d: toy_truth([3, 1, 4][: d % 3] + [first[d]], n_new) for d in range(n_dev)}
    for d in range(n_dev):
        s.open(d, prompt=[3, 1, 4][: d % 3])         # sessions may start from a prompt
    drafters = {d: serving.ReplayDrafter(truth[d], ToyShape.vocab, beta, seed=d) for d in range(n_dev)}
    res = serving.simulate(s, drafters, first, n_new, k, draft_ms_per_token=1.0, seed=1, lose_every=lose_every)
    assert res["devices_off_replayed_path"] == 0
    for d in range(n_dev):
        assert res["texts"][d] == truth[d]
        assert v.ctx[s.req_of[d]][: d % 3 + 1] == [3, 1, 4][: d % 3] + [first[d]]
    assert res["tokens"] == n_dev * n_new
    if beta == 1.0:
        assert res["accepted_per_draft"] == 1.0
        assert res["steps"] <= -(-n_dev // batch) * -(-n_new // (k + 1)) + n_dev
    if beta == 0.0:
        assert res["accepted_per_draft"] == 0.0 and res["steps"] == n_dev * n_new   # one token per device and step


def test_replay_drafter_statistics():
    truth = list(range(1000))
    d = serving.ReplayDrafter(truth, 5000, 0.75, seed=0)
    run = []
    for i in range(0, 900, 6):
        dr = d.draft(i, 6)
        n = 0
        while n < 6 and dr[n] == truth[i + n]:
            n += 1
        assert all(dr[j] != truth[i + j] for j in range(n, 6)) or n == 6 or dr[n] != truth[i + n]
        run.append(n)
    b = 0.75
    expect = b * (1 - b ** 6) / (1 - b)
    assert abs(np.mean(run) - expect) < 0.35
