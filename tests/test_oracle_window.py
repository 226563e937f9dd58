"""Pins for the oracle's TOPK with always-kept tokens (section 5, "Baselines and setup": the first
and the most recent tokens are always in context; the token budget counts only the retrieved ones).

Checked against a definition written here with Python sets and an exhaustive search, not against the
oracle's own routines.
"""
import itertools
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as W


def window_set_by_definition(scores, k, n_sink, n_local):
    """sink  u  best k of the tokens in between (score desc, index asc)  u  local."""
    n = len(scores)
    lo = min(n_sink, n)
    hi = max(lo, n - n_local)
    middle = sorted(range(lo, hi), key=lambda t: (-int(scores[t]), t))[:max(k, 0)]
    keep = set(range(lo)) | set(middle) | set(range(hi, n))
    return sorted(keep), middle


@pytest.mark.parametrize("n,k,s,l", [(40, 5, 4, 6), (40, 0, 4, 6), (40, 100, 4, 6), (9, 3, 4, 6), (10, 3, 4, 6),
                                     (11, 3, 4, 6), (1, 1, 0, 1), (0, 3, 2, 2), (25, 7, 0, 5), (25, 7, 5, 0)])
def test_window_equals_set_definition(n, k, s, l):
    rng = np.random.default_rng(1000 + n * 7 + k)
    for _ in range(20):
        sc = rng.integers(0, 5, size=n).astype(np.int32)       # few values: many ties
        idx, thr, got = oracle.topk_window(sc, k, s, l)
        want, middle = window_set_by_definition(sc, k, s, l)
        assert idx.tolist() == want
        assert got == len(middle)
        assert thr == (min(int(sc[t]) for t in middle) if middle else 0)
        assert len(set(idx.tolist())) == len(idx) and idx.tolist() == sorted(idx.tolist())


def test_window_exhaustive_tiny():
    """Every score vector over {0,1,2} of length 6 with sink 1, local 2: the retrieved part is the
    lexicographically smallest best subset of the middle (brute force over subsets)."""
    n, s, l, k = 6, 1, 2, 2
    mid = list(range(s, n - l))
    for sc in itertools.product(range(3), repeat=n):
        sc = np.array(sc, dtype=np.int32)
        best = None
        for sub in itertools.combinations(mid, k):
            key = (-sum(int(sc[t]) for t in sub), sub)       # highest total, then lowest ids
            # a k-subset is a valid top-k iff no outside middle token beats an inside one
            ok = all(sc[o] <= min(sc[t] for t in sub) for o in mid if o not in sub)
            if ok and (best is None or key < best[0]):
                best = (key, sub)
        idx, thr, got = oracle.topk_window(sc, k, s, l)
        assert got == k
        assert idx.tolist() == sorted(set(range(s)) | set(best[1]) | set(range(n - l, n)))


def test_no_window_is_plain_topk():
    rng = np.random.default_rng(5)
    for n, k in [(100, 10), (64, 64), (33, 40), (1, 1)]:
        sc = rng.integers(0, 33, size=n).astype(np.int32)
        idx, thr, got = oracle.topk_window(sc, k, 0, 0)
        ref, rthr = oracle.topk_sort(sc, k)
        assert idx.tolist() == ref.tolist() and thr == rthr and got == len(ref)


def test_budget_counts_only_retrieved_tokens():
    """Window tokens with the best scores do not use up the budget."""
    n, s, l, k = 300, 8, 16, 20
    rng = np.random.default_rng(6)
    sc = rng.integers(0, 20, size=n).astype(np.int32)
    sc[:s] = 32
    sc[n - l:] = 32
    idx, thr, got = oracle.topk_window(sc, k, s, l)
    assert got == k and len(idx) == s + k + l
    ref, _ = oracle.topk_sort(sc[s:n - l], k)
    assert idx[s:s + k].tolist() == (ref + s).tolist()
    assert thr <= 19


def test_window_covers_short_sequences_entirely():
    sc = np.arange(10, dtype=np.int32)
    for s, l in [(4, 6), (8, 8), (128, 128), (0, 10), (10, 0)]:
        idx, thr, got = oracle.topk_window(sc, 3, s, l)
        assert idx.tolist() == list(range(10)) and got == 0 and thr == 0


def test_count_formula():
    rng = np.random.default_rng(7)
    for _ in range(50):
        n = int(rng.integers(0, 400)); k = int(rng.integers(0, 60)); s = int(rng.integers(0, 140)); l = int(rng.integers(0, 140))
        sc = rng.integers(0, 33, size=n).astype(np.int32)
        idx, _, got = oracle.topk_window(sc, k, s, l)
        lo = min(s, n); hi = max(lo, n - l)
        assert got == min(k, hi - lo)
        assert len(idx) == lo + got + (n - hi)


def _small_layer(seed, n, batch=2):
    cfg = W.scaled(W.c1(context=n, k=8, batch=batch), name="win")
    return cfg, W.make_layer(cfg, seed)


def test_decode_step_window_composition_and_dense_limit():
    """decode_step with a window = its parts (scores -> window set -> gather_attend); a window that
    covers the whole sequence gives dense attention whatever the codes are (library SDPA, fp64)."""
    cfg, L = _small_layer(11, 96)
    g = cfg.group
    phi_q, phi_kv = oracle.Mlp(L.w_q), oracle.Mlp(L.w_kv)
    codes = np.zeros(L.k.shape[:3], dtype=np.uint32)
    cache = oracle.Cache(L.k, L.v, codes, L.seq_lens.copy())
    oracle.encode_keys(phi_kv, cache, None, None, int(L.seq_lens.max()))
    scale = 1.0 / math.sqrt(cfg.head_dim)
    kps = np.full(cfg.batch, 8, dtype=np.int32)
    res = oracle.decode_step(phi_q, phi_kv, cache, L.q, kps, scale, n_sink=5, n_local=7)
    assert res["idx"].shape[2] == 8 + 5 + 7
    for b in range(cfg.batch):
        n = int(L.seq_lens[b])
        for h in (0, 5, 31):
            sc = oracle.scores(int(res["q_codes"][b, h]), codes[b, h // g, :n])
            want, middle = window_set_by_definition(sc, 8, 5, 7)
            cnt = int(res["count"][b, h])
            assert res["idx"][b, h, :cnt].tolist() == want
            o = oracle.gather_attend(cache, b, h // g, L.q[b, h], np.array(want, dtype=np.int32), scale)
            np.testing.assert_allclose(res["out"][b, h], o, rtol=0, atol=1e-14)
    # whole sequence inside the window -> dense SDPA
    res = oracle.decode_step(phi_q, phi_kv, cache, L.q, kps, scale, n_sink=64, n_local=64)
    for b in range(cfg.batch):
        n = int(L.seq_lens[b])
        kf = torch.from_numpy(W.bf16_bits_to_f32(L.k[b, :, :n]).astype(np.float64))
        vf = torch.from_numpy(W.bf16_bits_to_f32(L.v[b, :, :n]).astype(np.float64))
        qf = torch.from_numpy(W.bf16_bits_to_f32(L.q[b]).astype(np.float64))
        for h in (0, 13, 31):
            ref = torch.nn.functional.scaled_dot_product_attention(
                qf[h][None, None], kf[h // g][None], vf[h // g][None], scale=scale)[0, 0].numpy()
            assert int(res["count"][b, h]) == n
            np.testing.assert_allclose(res["out"][b, h], ref, rtol=1e-10, atol=1e-12)
