"""GPU parity of hashattn_dense_attend (single-query SDPA over all cached tokens, section 3.1), the
in-house dense decode kernel every "sparse vs dense" figure is divided by, at the kinds of shape it is
timed on: GQA groups of 4 and 8, several splits per KV head with the split merge, ragged and empty
sequences, the paged layout with mixed lengths, and more than sixteen splits per head (both loops of
the merge).  Full-size sampled checks at the benchmark configurations are in test_gpu_full_size.py.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

gu = None


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    global gu
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import gpu_util
    gu = gpu_util
    yield


def check_dense(L, max_seq_len=None):
    """Every (sequence, query head) of the layer against oracle.dense_attend; returns the error summary."""
    D = gu.DeviceLayer(L)
    if max_seq_len is not None:
        D.cache.max_seq_len = max_seq_len            # a host bound above every actual length
    g = D.Hq // D.Hkv
    ocache, _, lens = D.oracle_cache()
    _, _, _, out = D.new_outputs()
    D.ctx.hashattn_dense_attend(D.q, D.cache, D.B, D.scale, out)
    torch.cuda.synchronize()
    ref = np.zeros((D.B, D.Hq, D.d))
    for b in range(D.B):
        for h in range(D.Hq):
            if lens[b] > 0:                          # an empty sequence gives a zero row
                ref[b, h] = oracle.dense_attend(ocache, b, h // g, L.q[b, h], int(lens[b]), D.scale)
    return gu.assert_out_close(out, ref, "dense_attend")


@pytest.mark.parametrize("group", [1, 2, 4, 8])
def test_dense_ragged_batch_contiguous(group):
    """Lengths 0, 1, one short of / exactly / one past a 64-row iteration, and several splits."""
    cfg = W.scaled(W.c1(), context=9001, k=16, batch=7, planted=4, n_q_heads=2 * group, n_kv_heads=2)
    L = W.make_layer(cfg, seed=71 + group)
    L.seq_lens[:] = [9001, 0, 1, 63, 64, 65, 4097]
    stats = check_dense(L)
    assert stats["same_bf16_frac"] > 0.9


def test_dense_llama_heads_many_sequences():
    """32 query heads on 8 KV heads, 20 sequences: the split shape taken for more than 128 (sequence, KV head) pairs."""
    cfg = W.scaled(W.c1(), context=6000, k=16, batch=20, planted=8)
    L = W.make_layer(cfg, seed=75)
    L.seq_lens[:] = 6000 - 293 * np.arange(20)
    check_dense(L)


def test_dense_host_bound_above_lengths():
    """seq_lens below the host's max_seq_len: the grid and the merge are sized by the bound, the work by the lengths."""
    cfg = W.scaled(W.c1(), context=5000, k=16, batch=3, planted=4)
    L = W.make_layer(cfg, seed=76)
    L.seq_lens[:] = [1200, 4999, 77]
    check_dense(L, max_seq_len=5000)


@pytest.mark.parametrize("group", [4, 8])
def test_dense_more_than_sixteen_splits(group):
    """One KV head, 40000 tokens: about 200 splits per head, so the merge runs its prefetched first
    sixteen partials, the unrolled loop and the tail."""
    cfg = W.scaled(W.c1(), context=40000, k=16, batch=1, planted=16, n_q_heads=group, n_kv_heads=1)
    L = W.make_layer(cfg, seed=77 + group)
    check_dense(L)


def test_dense_paged_mixed_lengths():
    """Page size 16, random page table, lengths log-uniform in [100, 9000] (the mixed-batch configuration, reduced)."""
    cfg = W.scaled(W.c4(batch=9, lo=100, hi=9000), planted=4)
    L = W.make_layer(cfg, seed=79)
    check_dense(L)


def test_dense_paged_group_of_eight():
    cfg = W.scaled(W.c4(batch=4, lo=50, hi=5000), planted=4, n_q_heads=16, n_kv_heads=2)
    L = W.make_layer(cfg, seed=80)
    check_dense(L)
