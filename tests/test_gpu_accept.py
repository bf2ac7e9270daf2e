"""GPU parity of sled_accept against the oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

from paper_2506_09397_amd import sled, synth
from gpu_common import compare_accept, oracle_accept, run_accept_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("vocab,k", [
    (1024, [4, 4, 4, 4]),
    (1000, [0, 3, 8, 1, 0, 5]),        # vocab not a multiple of the vector width, k = 0 requests
    (4099, [8] * 7),                    # odd vocab: scalar path, several tiles + ragged tail in the draw
    (32000, [2, 4, 6, 8] * 8),
    (130, [1, 2]),
])
@pytest.mark.parametrize("sigma", [0.25, 1.0, 4.0])
def test_sampling_matches_oracle_small(vocab, k, sigma):
    case = synth.accept_case(k, vocab, sigma, seed=vocab + int(sigma * 10), device="cuda")
    a, t = run_accept_gpu(sled.SAMPLE, case, vocab)
    want = oracle_accept(sled.SAMPLE, case)
    n_sub = compare_accept(sled.SAMPLE, k, a, t, want, f"V={vocab} sigma={sigma}")
    assert n_sub <= 1


@pytest.mark.parametrize("vocab,k", [(1024, [4, 4, 4, 4]), (1000, [0, 3, 8, 1]), (128256, [2, 8, 5, 3, 7, 4] * 3)])
def test_greedy_matches_oracle(vocab, k):
    case = synth.accept_case(k, vocab, 0.25, seed=5, device="cuda")
    # make about half of the drafts equal to the target argmax so that accepted lengths vary
    logits = case.logits
    off = 0
    g = torch.Generator(device="cuda").manual_seed(1)
    for ki in k:
        for j in range(ki):
            if torch.rand(1, generator=g, device="cuda").item() < 0.7:
                case.tokens[off + 1 + j] = int(torch.argmax(logits[off + j]))
        off += ki + 1
    a, t = run_accept_gpu(sled.GREEDY, case, vocab)
    want = oracle_accept(sled.GREEDY, case)
    assert compare_accept(sled.GREEDY, k, a, t, want) == 0
    assert max(int(x) for x in a) > 0


@pytest.mark.parametrize("mode", ["greedy", "sample"])
def test_long_drafts_fail_beyond_the_first_wavefront_pass(mode):
    """k up to the maximum of 255: the deciding wavefront judges 64 rows per pass, so the first
    failure is put at draft 0, inside the first pass, on a pass boundary, deep in a later pass, and nowhere."""
    vocab = 512
    k = [255, 200, 130, 64, 65, 255, 3]
    fail_at = [0, 37, 64, 63, None, 254, None]     # index of the first rejected draft
    case = synth.accept_case(k, vocab, 0.0, seed=9, device="cuda")   # sigma 0: q == p, every draft passes Eq. 1
    off = doff = 0
    for ki, f in zip(k, fail_at):
        rows = slice(off, off + ki)
        if mode == "greedy":
            case.tokens[off + 1: off + 1 + ki] = torch.argmax(case.logits[rows], dim=1).int()
            if f is not None:
                case.tokens[off + 1 + f] = (case.tokens[off + 1 + f] + 1) % vocab
        elif f is not None:
            # draft probability 1 for a token the target gives about 1/512: rejected for u = 0.9
            d = int(case.tokens[off + 1 + f])
            case.q[doff + f].zero_()
            case.q[doff + f, d] = 1.0
            case.u_acc[doff + f] = 0.9
        off += ki + 1
        doff += ki
    m = sled.GREEDY if mode == "greedy" else sled.SAMPLE
    a, t = run_accept_gpu(m, case, vocab)
    want = oracle_accept(m, case)
    assert [w["accept_len"] for w in want] == [ki if f is None else f for ki, f in zip(k, fail_at)]
    assert compare_accept(m, k, a, t, want, mode) <= (0 if mode == "greedy" else 1)
    assert a.tolist() == [w["accept_len"] for w in want]


def test_greedy_ties_take_lowest_id():
    vocab, k = 4096, [3, 2]
    T = sum(k) + len(k)
    g = torch.Generator(device="cuda").manual_seed(3)
    logits = torch.randint(0, 4, (T, vocab), generator=g, device="cuda").float()   # many exact ties
    tokens = torch.zeros(T, dtype=torch.int32, device="cuda")
    first_max = torch.argmax((logits == logits.max(dim=1, keepdim=True).values).float(), dim=1)
    tokens[1:4] = first_max[0:3].int()
    tokens[5] = first_max[4].int()
    tokens[6] = (first_max[5] + 1).int()     # wrong on purpose
    case = synth.AcceptCase(k, logits, tokens, None, None, None)
    a, t = run_accept_gpu(sled.GREEDY, case, vocab)
    assert a.tolist() == [3, 1]
    assert t.tolist() == [int(first_max[3]), int(first_max[5])]


@pytest.mark.parametrize("temperature", [0.7, 2.0])
def test_sampling_with_temperature(temperature):
    vocab, k = 5000, [4, 3, 8, 0, 2]
    case = synth.accept_case(k, vocab, 1.0, seed=17, device="cuda")
    a, t = run_accept_gpu(sled.SAMPLE, case, vocab, temperature)
    want = oracle_accept(sled.SAMPLE, case, temperature)
    assert compare_accept(sled.SAMPLE, k, a, t, want) <= 1


@pytest.mark.parametrize("sigma", [0.25, 1.0, 4.0])
def test_acceptance_alone_full_size(sigma):
    """256 requests x (8 drafts + 1 bonus row) x vocab 128256, target logits N(0, 2)."""
    vocab, k = 128256, [8] * 256
    case = synth.accept_case(k, vocab, sigma, seed=int(sigma * 100), device="cuda")
    a, t = run_accept_gpu(sled.SAMPLE, case, vocab)
    want = oracle_accept(sled.SAMPLE, case)
    n_sub = compare_accept(sled.SAMPLE, k, a, t, want, f"sigma={sigma}")
    assert n_sub <= 3
    mean_a = float(np.mean(a))
    # acceptance falls as the draft distribution moves away from the target
    lo, hi = {0.25: (3.5, 7.0), 1.0: (0.8, 2.8), 4.0: (0.0, 0.4)}[sigma]
    assert lo <= mean_a <= hi, mean_a


def _sparse_case(k, vocab, m, sigma, seed, pad=0):
    """Drafts drawn from the top-m tokens (renormalised) of softmax(target row + sigma * noise); returns the case
    with the dense truncated q (for the oracle) and the (ids, probs) pairs, `pad` padding entries appended."""
    case = synth.accept_case(k, vocab, sigma, seed=seed, device="cuda")
    top = torch.topk(case.q, m, dim=1)
    probs = (top.values / top.values.sum(dim=1, keepdim=True)).float()
    ids = top.indices.int()
    g = torch.Generator(device="cuda").manual_seed(seed + 1)
    pick = torch.multinomial(probs, 1, generator=g).squeeze(1)
    drafts = ids[torch.arange(ids.shape[0], device="cuda"), pick]
    off = doff = 0
    for ki in k:
        case.tokens[off + 1: off + 1 + ki] = drafts[doff: doff + ki]
        off += ki + 1
        doff += ki
    dense = torch.zeros_like(case.q)
    dense.scatter_(1, ids.long(), probs)
    case.q = dense
    if pad:
        ids = torch.cat([ids, torch.full((ids.shape[0], pad), -1, dtype=torch.int32, device="cuda")], dim=1)
        probs = torch.cat([probs, torch.zeros(probs.shape[0], pad, device="cuda")], dim=1)
        # padding may sit anywhere in a row
        perm = torch.randperm(ids.shape[1], generator=g, device="cuda")
        ids, probs = ids[:, perm].contiguous(), probs[:, perm].contiguous()
    return case, ids.contiguous(), probs.contiguous()


def _run_sparse(case, vocab, ids, probs, temperature=1.0):
    B, T = len(case.k), sum(case.k) + len(case.k)
    ws = sled.workspace(sled.sled_accept_workspace_bytes(B, T, vocab))
    a = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    t = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    sled.sled_accept_sparse(case.k, vocab, temperature, case.logits, case.tokens, ids, probs, case.u_acc, case.u_smp, a, t, ws)
    torch.cuda.synchronize()
    return a.cpu().numpy(), t.cpu().numpy()


@pytest.mark.parametrize("vocab,k,m,pad", [
    (1024, [4, 4, 4, 4], 8, 0),
    (4099, [8, 0, 3, 5, 1], 64, 5),        # odd vocabulary, padding entries
    (32000, [2, 4, 6, 8] * 4, 256, 0),
    (128256, [2, 8, 5, 3, 7, 4] * 3, 64, 0),
    (1000, [6, 6, 6], 1, 0),               # one-hot q: a greedy drafter
    (5000, [3] * 5, 1024, 0),              # the largest row the entry point takes
])
@pytest.mark.parametrize("sigma", [0.5, 2.0])
def test_sparse_draft_distributions_match_oracle(vocab, k, m, pad, sigma):
    case, ids, probs = _sparse_case(k, vocab, m, sigma, seed=vocab + m, pad=pad)
    a, t = _run_sparse(case, vocab, ids, probs)
    want = oracle_accept(sled.SAMPLE, case)
    n_sub = compare_accept(sled.SAMPLE, k, a, t, want, f"V={vocab} m={m} sigma={sigma}")
    assert n_sub <= 1
    # and the dense entry point, given the same truncated q, agrees
    a2, t2 = run_accept_gpu(sled.SAMPLE, case, vocab)
    assert compare_accept(sled.SAMPLE, k, a2, t2, want) <= 1


@pytest.mark.parametrize("vocab,k,m,pad", [
    (1024, [4, 4, 4, 4], 8, 0),
    (4099, [8, 0, 3, 5, 1], 64, 5),        # odd vocabulary, padding entries
    (32000, [2, 4, 6, 8] * 4, 256, 0),
    (128256, [2, 8, 5, 3, 7, 4] * 3, 64, 0),
    (1000, [6, 6, 6], 1, 0),               # one listed token and the rest of the mass on everything else
])
@pytest.mark.parametrize("sigma", [0.5, 2.0])
def test_sparse_draft_distributions_with_remainder_mass_match_oracle(vocab, k, m, pad, sigma):
    """Top-m pairs as the drafter had them plus the mass of everything else, spread evenly over the unlisted tokens:
    the library given (ids, probabilities, remainder) against the oracle given the reconstructed dense distribution;
    drafts are drawn from that reconstruction, so some of them are unlisted tokens."""
    case = synth.accept_case(k, vocab, sigma, seed=vocab + m + 1, device="cuda")
    top = torch.topk(case.q, m, dim=1)
    ids, probs = top.indices.int(), top.values.float().clone()
    rest = (1.0 - probs.double().sum(dim=1)).clamp_min(0.0).float()
    dense = (rest / (vocab - m))[:, None].expand(-1, vocab).clone()
    dense.scatter_(1, ids.long(), probs)
    g = torch.Generator(device="cuda").manual_seed(vocab + 7)
    drafts = torch.multinomial(dense.double(), 1, generator=g).squeeze(1)
    off = doff = 0
    for ki in k:
        case.tokens[off + 1: off + 1 + ki] = drafts[doff: doff + ki].int()
        off += ki + 1
        doff += ki
    case.q = dense
    if pad:
        ids = torch.cat([ids, torch.full((ids.shape[0], pad), -1, dtype=torch.int32, device="cuda")], dim=1)
        probs = torch.cat([probs, torch.zeros(probs.shape[0], pad, device="cuda")], dim=1)
        perm = torch.randperm(ids.shape[1], generator=g, device="cuda")
        ids, probs = ids[:, perm], probs[:, perm]
    ids, probs = ids.contiguous(), probs.contiguous()
    B, T = len(k), sum(k) + len(k)
    ws = sled.workspace(sled.sled_accept_workspace_bytes(B, T, vocab))
    a = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    t = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    sled.sled_accept_sparse(k, vocab, 1.0, case.logits, case.tokens, ids, probs, case.u_acc, case.u_smp, a, t, ws, q_rest=rest)
    torch.cuda.synchronize()
    want = oracle_accept(sled.SAMPLE, case)
    n_sub = compare_accept(sled.SAMPLE, k, a.cpu().numpy(), t.cpu().numpy(), want, f"V={vocab} m={m} sigma={sigma} with remainder")
    assert n_sub <= 1
    n_off = sum(int(d) not in set(r.tolist()) for d, r in zip(drafts.cpu(), top.indices.cpu()))
    assert m >= 64 or n_off > 0          # the short lists leave enough mass off the list for unlisted drafts to occur


def test_sparse_token_outside_its_row_is_accepted_and_errors():
    vocab, k = 2048, [3, 2]
    case, ids, probs = _sparse_case(k, vocab, 16, 1.0, seed=3)
    # a draft that its own row does not list has q = 0: the product form of Eq. 1 accepts it
    outside = [t for t in range(vocab) if t not in set(ids[0].tolist())][0]
    case.tokens[1] = outside
    a, t = _run_sparse(case, vocab, ids, probs)
    want = oracle_accept(sled.SAMPLE, case)
    assert want[0]["accept_len"] >= 1
    assert compare_accept(sled.SAMPLE, k, a, t, want) <= 1
    ws = sled.workspace(sled.sled_accept_workspace_bytes(2, 7, vocab))
    o = torch.zeros(2, dtype=torch.int32, device="cuda")
    big_i = torch.zeros(5, 1025, dtype=torch.int32, device="cuda")
    with pytest.raises(sled.SledError):
        sled.sled_accept_sparse(k, vocab, 1.0, case.logits, case.tokens, big_i, big_i.float(), case.u_acc, case.u_smp, o, o.clone(), ws)
    with pytest.raises(sled.SledError):
        sled.sled_accept_sparse(k, vocab, 0.0, case.logits, case.tokens, ids, probs, case.u_acc, case.u_smp, o, o.clone(), ws)


@pytest.mark.parametrize("sparse", [False, True])
def test_draft_outside_the_vocabulary_is_rejected_not_read(sparse):
    """Draft ids come from the devices: one outside [0, V) ends the accepted prefix at its position (dense and
    sparse q, and greedy), and is never used as an index."""
    vocab, k = 2048, [4, 3, 5, 2]
    if sparse:
        case, ids, probs = _sparse_case(k, vocab, 16, 0.0, seed=11)
    else:
        case = synth.accept_case(k, vocab, 0.0, seed=11, device="cuda")      # q == p: every in-vocabulary draft passes
    case.u_acc.zero_()                                                       # ... and so does every draft of a truncated q
    bad = {0: (2, -1), 1: (0, vocab), 2: (4, 2**31 - 1), 3: (1, -(2**31))}     # request -> (draft index, bad id)
    off = 0
    for i, ki in enumerate(k):
        j, v = bad[i]
        case.tokens[off + 1 + j] = v
        off += ki + 1
    a, t = _run_sparse(case, vocab, ids, probs) if sparse else run_accept_gpu(sled.SAMPLE, case, vocab)
    want = oracle_accept(sled.SAMPLE, case)
    assert [w["accept_len"] for w in want] == [bad[i][0] for i in range(len(k))]
    assert compare_accept(sled.SAMPLE, k, a, t, want) <= 1
    assert [int(x) for x in a] == [bad[i][0] for i in range(len(k))]
    g, tg = run_accept_gpu(sled.GREEDY, case, vocab)
    wg = oracle_accept(sled.GREEDY, case)
    assert compare_accept(sled.GREEDY, k, g, tg, wg) == 0 and all(int(g[i]) <= bad[i][0] for i in range(len(k)))


def test_accept_argument_errors():
    vocab, k = 1024, [2, 2]
    case = synth.accept_case(k, vocab, 1.0, seed=1, device="cuda")
    a = torch.zeros(2, dtype=torch.int32, device="cuda")
    ws = sled.workspace(sled.sled_accept_workspace_bytes(2, 6, vocab))
    with pytest.raises(sled.SledError) as e:
        sled.sled_accept(5, k, vocab, 1.0, case.logits, case.tokens, case.q, case.u_acc, case.u_smp, a, a.clone(), ws)
    assert e.value.code == sled.EINVAL
    with pytest.raises(sled.SledError):
        sled.sled_accept(sled.SAMPLE, k, vocab, 0.0, case.logits, case.tokens, case.q, case.u_acc, case.u_smp, a, a.clone(), ws)
    with pytest.raises(sled.SledError):
        sled.sled_accept(sled.SAMPLE, k, vocab, 1.0, case.logits, case.tokens, None, case.u_acc, case.u_smp, a, a.clone(), ws)
    with pytest.raises(sled.SledError):
        sled.sled_accept(sled.SAMPLE, k, vocab, 1.0, case.logits, case.tokens, case.q, case.u_acc, case.u_smp, a, a.clone(),
                         ws[:64])


@pytest.mark.parametrize("T,vocab,temperature,std", [
    (1, 130, 1.0, 2.0),
    (37, 1000, 0.7, 2.0),             # vocab not a multiple of the vector width
    (9, 4099, 1.0, 4.0),              # odd vocab: scalar path
    (101, 128256, 1.0, 1.28),         # the headline step's logits shape, logits of the random-weight model's scale
    (2304, 128256, 2.0, 2.0),         # 256 requests x 9 rows: one segment per row
])
def test_row_confidence_matches_oracle(T, vocab, temperature, std):
    """sled_row_confidence (the score Eq. 2 thresholds) against the oracle's float64 softmax: the token exactly
    (unless the two best logits are closer than float32 resolves -- none at these seeds), the probability to
    1e-5 relative (float32 exponentials, float64 sums)."""
    from oracle import sled_oracle as O
    g = torch.Generator(device="cuda").manual_seed(T * 7 + vocab)
    logits = torch.randn(T, vocab, generator=g, device="cuda", dtype=torch.float32) * std
    logits[0, min(5, vocab - 1)] = logits[0].max() + 3.0          # one confident row
    if T > 2:
        logits[2, :] = 0.125                                      # a row of equal logits: 1/V, token 0
    conf = torch.empty(T, dtype=torch.float32, device="cuda")
    top = torch.empty(T, dtype=torch.int32, device="cuda")
    ws = sled.workspace(sled.sled_accept_workspace_bytes(1, T, vocab))
    sled.sled_row_confidence(vocab, temperature, logits, conf, top, ws)
    torch.cuda.synchronize()
    rows = range(T) if T <= 128 else list(range(0, T, 97)) + [T - 1]
    want_c, want_t = O.row_confidence(logits[list(rows)].cpu().numpy().astype(np.float64), temperature)
    got_c, got_t = conf.cpu().numpy()[list(rows)], top.cpu().numpy()[list(rows)]
    assert (got_t == want_t).all()
    assert np.abs(got_c / want_c - 1.0).max() < 1e-5
    if T > 2:
        assert top[2].item() == 0 and abs(conf[2].item() * vocab - 1.0) < 1e-5
    # the token is optional
    conf2 = torch.empty_like(conf)
    sled.sled_row_confidence(vocab, temperature, logits, conf2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(conf, conf2)


def test_row_confidence_argument_errors():
    logits = torch.zeros(4, 256, device="cuda")
    conf = torch.empty(4, device="cuda")
    ws = sled.workspace(sled.sled_accept_workspace_bytes(1, 4, 256))
    with pytest.raises(sled.SledError):
        sled.sled_row_confidence(256, 0.0, logits, conf, None, ws)          # temperature
    with pytest.raises(sled.SledError):
        sled.sled_row_confidence(1, 1.0, logits, conf, None, ws)            # vocabulary
    with pytest.raises(sled.SledError):
        sled.sled_row_confidence(256, 1.0, logits, conf, None, ws[:64])     # workspace too small
