"""Pins for the oracle's quality measures: recall(I_n, I_true,k) (section 4) and the true pivotal
tokens ranked by a_i * ||v_i||_2 (lemma of section 4.2), against formulas written here with numpy /
torch in fp64 and against hand cases."""
import math

import numpy as np
import torch

import oracle
import workloads as W


def _layer(seed, n=200, batch=1):
    cfg = W.scaled(W.c1(context=n, k=8, batch=batch), name="recall")
    L = W.make_layer(cfg, seed)
    codes = np.zeros(L.k.shape[:3], dtype=np.uint32)
    return cfg, L, oracle.Cache(L.k, L.v, codes, L.seq_lens.copy())


def test_recall_hand_cases():
    t = np.array([3, 9, 27, 81], dtype=np.int32)
    assert oracle.recall(np.array([3, 9, 27, 81], dtype=np.int32), t) == 1.0
    assert oracle.recall(np.array([81, 5, 3], dtype=np.int32), t) == 0.5
    assert oracle.recall(np.array([1, 2, 4], dtype=np.int32), t) == 0.0
    assert oracle.recall(np.array([], dtype=np.int32), t) == 0.0
    assert oracle.recall(np.arange(50, dtype=np.int32), t) == 0.75            # 3, 9 and 27 of the four
    rng = np.random.default_rng(1)
    for _ in range(50):
        a = rng.choice(500, size=int(rng.integers(0, 60)), replace=False).astype(np.int32)
        b = rng.choice(500, size=int(rng.integers(1, 60)), replace=False).astype(np.int32)
        want = len(set(a.tolist()) & set(b.tolist())) / len(b)
        assert oracle.recall(a, b) == want
        assert oracle.recall(rng.permutation(a).astype(np.int32), rng.permutation(b).astype(np.int32)) == want


def test_contributions_equal_norm_of_the_single_token_term():
    """a_i ||v_i|| is the Euclidean norm of token i's term a_i v_i of the dense output (fp64 torch)."""
    cfg, L, cache = _layer(3)
    g, n, scale = cfg.group, 200, 1.0 / math.sqrt(128)
    for h in (0, 7, 31):
        kf = torch.from_numpy(W.bf16_bits_to_f32(L.k[0, h // g, :n]).astype(np.float64))
        vf = torch.from_numpy(W.bf16_bits_to_f32(L.v[0, h // g, :n]).astype(np.float64))
        qf = torch.from_numpy(W.bf16_bits_to_f32(L.q[0, h]).astype(np.float64))
        a = torch.softmax(kf @ qf * scale, dim=0)
        want = torch.linalg.vector_norm(a[:, None] * vf, dim=1).numpy()
        got = oracle.token_contributions(cache, 0, h // g, L.q[0, h], n, scale)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-300)
        # the terms add up to the dense output
        dense = oracle.dense_attend(cache, 0, h // g, L.q[0, h], n, scale)
        np.testing.assert_allclose((a[:, None] * vf).sum(0).numpy(), dense, rtol=1e-10, atol=1e-13)


def test_true_topk_is_the_sorted_prefix_and_v_norm_matters():
    cfg, L, cache = _layer(4)
    g, n, scale = cfg.group, 200, 1.0 / math.sqrt(128)
    h = 5
    contrib = oracle.token_contributions(cache, 0, h // g, L.q[0, h], n, scale)
    for k in (1, 7, 64, 200, 500):
        want = sorted(sorted(range(n), key=lambda t: (-contrib[t], t))[:k])
        assert oracle.true_topk(cache, 0, h // g, L.q[0, h], n, k, scale).tolist() == want
    # blowing up one value row promotes that token; the attention weights alone would not
    weak = int(np.argsort(contrib)[n // 2])
    assert weak not in oracle.true_topk(cache, 0, h // g, L.q[0, h], n, 4, scale).tolist()
    v2 = L.v.copy()
    v2[0, h // g, weak] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(v2[0, h // g, weak]) * 4096.0)
    cache2 = oracle.Cache(L.k, v2, np.zeros(L.k.shape[:3], dtype=np.uint32), L.seq_lens.copy())
    assert weak in oracle.true_topk(cache2, 0, h // g, L.q[0, h], n, 4, scale).tolist()


def test_planted_tokens_are_the_true_pivotal_tokens():
    """The workload plants keys aligned with the query: they carry the attention mass."""
    cfg = W.scaled(W.c1(context=2048, k=64), name="planted")
    L = W.make_layer(cfg, 9)
    cache = oracle.Cache(L.k, L.v, np.zeros(L.k.shape[:3], dtype=np.uint32), L.seq_lens.copy())
    scale = 1.0 / math.sqrt(128)
    for h in (0, 13, 31):
        truth = oracle.true_topk(cache, 0, h // cfg.group, L.q[0, h], 2048, 32, scale)
        planted = L.planted_pos[0, h]
        assert oracle.recall(planted.astype(np.int32), truth) >= 0.9
