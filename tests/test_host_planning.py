"""Host-side planning of a verification step, through the C ABI, without a GPU.

Two choices are made on the host for every step: how the attention over requests of different lengths (Sec. 3.4: one
batch of heterogeneous requests) is cut into work items, and how many K slices each projection runs with.  Both are
exported as planning aids (sled_attention_partition, sled_projection_slices); here their contracts are checked:
the limits the header states, and that the partition never loses to the two simple rules it replaced."""
import numpy as np
import pytest

from paper_2506_09397_amd import sled, synth

CUS = 256


def _items(n_pages, tgt, H):
    """sizes of the work items of one launch, in launch order (longest requests first, even split per request)"""
    out = []
    for n in sorted(n_pages, reverse=True):
        pieces = -(-n // tgt)
        chunk = -(-n // pieces)
        sizes = [min(chunk, n - p0) for p0 in range(0, n, chunk)]
        assert len(sizes) == pieces
        out += sizes * H
    return out


def _pages(kind, shape):
    b = synth.draw_batch(kind, synth.SHAPES[shape].vocab, seed=0)
    return [-(-(int(L) + int(k) + 1) // 16) for L, k in zip(b.ctx_len, b.k)], synth.SHAPES[shape].n_kv_heads


@pytest.mark.parametrize("kind,shape", [("b16", "llama8b"), ("hetero64", "llama8b"), ("b32", "llama70b"), ("tiny4", "tiny_bf16")])
def test_partition_keeps_its_limits_on_the_benchmark_batches(kind, shape):
    n_pages, H = _pages(kind, shape)
    tgt, n_items = sled.sled_attention_partition(H, n_pages)
    sizes = _items(n_pages, tgt, H)
    assert n_items == len(sizes) and sum(sizes) == H * sum(n_pages)          # every page of every head exactly once
    longest = max(n_pages)
    assert 1 <= tgt <= longest
    for n in n_pages:
        pieces = -(-n // tgt)
        assert pieces <= 8
        if pieces > 1:
            assert n // pieces >= 16          # halves of at least 32 pages, split evenly
            assert tgt >= 32
    base = CUS * -(-len(n_pages) * H // CUS)
    assert n_items <= 4 * base


def test_partition_splits_the_long_requests_of_a_mixed_batch_and_leaves_an_even_batch_alone():
    n_pages, H = _pages("hetero64", "llama8b")
    tgt, n_items = sled.sled_attention_partition(H, n_pages)
    assert tgt < max(n_pages) and n_items > H * len(n_pages)      # the 8192-token request does not stay one item per head
    # the busiest CU's share: no worse than leaving every request whole
    assert max(_items(n_pages, tgt, H)) < max(n_pages)
    # 32 requests of one length on 8 heads: 256 equal items, nothing to gain from cutting them
    tgt, n_items = sled.sled_attention_partition(8, [100] * 32)
    assert (tgt, n_items) == (100, 256)
    # one long request alone: cut into the most items the limits allow (eight per head)
    tgt, n_items = sled.sled_attention_partition(8, [4096])
    assert n_items == 64 and tgt == 512
    # a request shorter than 32 pages is never cut
    tgt, n_items = sled.sled_attention_partition(8, [20, 31, 7])
    assert n_items == 24


def test_partition_on_random_batches():
    rng = np.random.default_rng(0)
    for _ in range(60):
        B = int(rng.integers(1, 97))
        H = int(rng.choice([1, 2, 8]))
        n_pages = [int(x) for x in np.exp(rng.uniform(np.log(1), np.log(600), size=B)).astype(int) + 1]
        tgt, n_items = sled.sled_attention_partition(H, n_pages)
        sizes = _items(n_pages, tgt, H)
        assert n_items == len(sizes) and sum(sizes) == H * sum(n_pages)
        assert all(-(-n // tgt) <= 8 for n in n_pages)
        assert all(n <= tgt or tgt >= 32 for n in n_pages)
        assert n_items <= 4 * CUS * -(-B * H // CUS)


def test_partition_rejects_bad_arguments():
    with pytest.raises(Exception):
        sled.sled_attention_partition(8, [0, 5])
    with pytest.raises(Exception):
        sled.sled_attention_partition(0, [5])


def test_projection_slices_of_the_benchmark_model():
    d, F, nqkv = 4096, 14336, (32 + 2 * 8) * 128
    # one block of rows (up to 128): the model's plan
    assert sled.sled_projection_slices(nqkv, d, 101) == (4, 8)
    assert sled.sled_projection_slices(d, d, 101) == (8, 16)
    assert sled.sled_projection_slices(d, F, 101) == (8, 16)
    assert sled.sled_projection_slices(2 * F, d, 101) == (1, 1)      # gate/up: enough column blocks, SwiGLU in the epilogue
    # three blocks of rows: whole rounds of 256 workgroups (24 x 3 x 3 = 216, 16 x 3 x 5 = 240)
    assert sled.sled_projection_slices(nqkv, d, 372)[0] == 3
    assert sled.sled_projection_slices(d, d, 372)[0] == 5
    assert sled.sled_projection_slices(d, F, 372)[0] == 5
    for N, K in ((nqkv, d), (d, d), (d, F), (10240, 8192), (8192, 28672)):
        for T in (1, 33, 128, 129, 225, 372, 512, 1008, 2016, 4096):
            s, cap = sled.sled_projection_slices(N, K, T)
            assert 1 <= s <= cap and s <= K // 256        # every slice holds at least one trip of the stage loop
            if T <= 128:
                assert s == sled.sled_projection_slices(N, K, 1)[0]
    with pytest.raises(Exception):
        sled.sled_projection_slices(100, 4096, 10)
