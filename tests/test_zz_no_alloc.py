"""sled_accept_static (the entry point that allocates nothing: its scratch is a fixed array inside the library) against
sled_accept on the same inputs, through the C ABI: two calls in a row, the second with a smaller input, greedy and
sampling; and the size limit."""
import pytest
import torch

from paper_2506_09397_amd import sled, synth

pytestmark = pytest.mark.gpu


def _both(mode, case, vocab):
    B, T = len(case.k), sum(case.k) + len(case.k)
    q, ua, us = (case.q, case.u_acc, case.u_smp) if mode == sled.SAMPLE else (None, None, None)
    ws = sled.workspace(sled.sled_accept_workspace_bytes(B, T, vocab))
    a0 = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    t0 = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    sled.sled_accept(mode, case.k, vocab, 1.0, case.logits, case.tokens, q, ua, us, a0, t0, ws)
    a1 = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    t1 = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    sled.sled_accept_static(mode, case.k, vocab, 1.0, case.logits, case.tokens, q, ua, us, a1, t1)
    torch.cuda.synchronize()
    return (a0.cpu(), t0.cpu()), (a1.cpu(), t1.cpu())


@pytest.mark.parametrize("mode", [sled.GREEDY, sled.SAMPLE])
def test_static_scratch_entry_point_equals_sled_accept_twice_in_a_row(mode):
    vocab = 32000
    big = synth.accept_case([8, 3, 0, 6, 8, 1, 5, 8] * 4, vocab, 1.0, seed=31, device="cuda")    # 188 rows
    small = synth.accept_case([2, 0, 4], vocab, 0.25, seed=32, device="cuda")                     # 9 rows, more segments per row
    for case in (big, small):     # the second call finds the first one's statistics in the array
        (a0, t0), (a1, t1) = _both(mode, case, vocab)
        assert torch.equal(a0, a1) and torch.equal(t0, t1)
        assert int(a0.min()) >= 0 and int(t0.min()) >= 0


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    vocab = 64
    k = [255] * 65                                   # 16640 rows > 16384
    T = sum(k) + len(k)
    logits = torch.zeros(T, vocab, device="cuda")
    tokens = torch.zeros(T, dtype=torch.int32, device="cuda")
    o = torch.zeros(len(k), dtype=torch.int32, device="cuda")
    with pytest.raises(sled.SledError) as e:
        sled.sled_accept_static(sled.GREEDY, k, vocab, 1.0, logits, tokens, None, None, None, o, o.clone())
    assert e.value.code == sled.EINVAL and "static scratch" in str(e.value)
    with pytest.raises(sled.SledError):
        sled.sled_accept_static(sled.SAMPLE, [2], vocab, 1.0, logits, tokens, None, None, None, o, o.clone())
