"""Pins for the oracle's GATHER-ATT (section 4) and single-query SDPA (section 3.1).

Checked against torch's CPU scaled_dot_product_attention (a library routine),
and against special cases with known answers: one selected token, equal keys,
permutation and shift invariance, the convex-hull bound, paged vs contiguous.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as W


def make_cache(rng, B, H, N, d=128, scale=1.0):
    k = W.f32_to_bf16_bits(rng.standard_normal((B, H, N, d), dtype=np.float32) * scale)
    v = W.f32_to_bf16_bits(rng.standard_normal((B, H, N, d), dtype=np.float32))
    codes = np.zeros((B, H, N), dtype=np.uint32)
    lens = np.full(B, N, dtype=np.int32)
    return oracle.Cache(k, v, codes, lens), k, v


def test_all_tokens_equals_library_sdpa():
    rng = np.random.default_rng(10)
    B, H, N, d = 2, 3, 257, 128
    cache, k, v = make_cache(rng, B, H, N)
    q = W.f32_to_bf16_bits(rng.standard_normal((B, H, d), dtype=np.float32))
    scale = 1.0 / math.sqrt(d)
    kt = torch.from_numpy(W.bf16_bits_to_f32(k)).double()
    vt = torch.from_numpy(W.bf16_bits_to_f32(v)).double()
    qt = torch.from_numpy(W.bf16_bits_to_f32(q)).double().unsqueeze(2)     # [B,H,1,d]
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt).squeeze(2).numpy()
    for b in range(B):
        for h in range(H):
            dense = oracle.dense_attend(cache, b, h, q[b, h], N, scale)
            full = oracle.gather_attend(cache, b, h, q[b, h], np.arange(N, dtype=np.int32), scale)
            np.testing.assert_allclose(dense, ref[b, h], rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(full, ref[b, h], rtol=1e-10, atol=1e-12)


def test_subset_equals_library_sdpa_on_gathered_rows():
    rng = np.random.default_rng(11)
    B, H, N, d = 1, 2, 500, 128
    cache, k, v = make_cache(rng, B, H, N, scale=2.0)
    q = W.f32_to_bf16_bits(rng.standard_normal((B, H, d), dtype=np.float32))
    idx = np.sort(rng.choice(N, size=37, replace=False)).astype(np.int32)
    for scale in (1.0 / math.sqrt(d), 0.31):
        for h in range(H):
            kt = torch.from_numpy(W.bf16_bits_to_f32(k[0, h, idx])).double()[None, None]
            vt = torch.from_numpy(W.bf16_bits_to_f32(v[0, h, idx])).double()[None, None]
            qt = torch.from_numpy(W.bf16_bits_to_f32(q[0, h])).double()[None, None, None]
            ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, scale=scale)[0, 0, 0].numpy()
            got = oracle.gather_attend(cache, 0, h, q[0, h], idx, scale)
            np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)


def test_single_token_returns_its_value_row():
    rng = np.random.default_rng(12)
    cache, k, v = make_cache(rng, 1, 1, 50)
    q = W.f32_to_bf16_bits(rng.standard_normal(128, dtype=np.float32))
    for i in (0, 7, 49):
        out = oracle.gather_attend(cache, 0, 0, q, np.array([i], dtype=np.int32), 0.1)
        np.testing.assert_array_equal(out, W.bf16_bits_to_f32(v[0, 0, i]).astype(np.float64))


def test_equal_keys_give_plain_mean_and_hull_bound():
    rng = np.random.default_rng(13)
    cache, k, v = make_cache(rng, 1, 1, 64)
    k[0, 0, :] = k[0, 0, 0]                     # all keys identical -> uniform weights
    q = W.f32_to_bf16_bits(rng.standard_normal(128, dtype=np.float32))
    idx = np.array([3, 9, 10, 40], dtype=np.int32)
    out = oracle.gather_attend(cache, 0, 0, q, idx, 0.5)
    vf = W.bf16_bits_to_f32(v[0, 0, idx]).astype(np.float64)
    np.testing.assert_allclose(out, vf.mean(axis=0), rtol=1e-12, atol=1e-14)
    # general keys: each coordinate is a convex combination of the gathered values
    cache2, k2, v2 = make_cache(rng, 1, 1, 64)
    out2 = oracle.gather_attend(cache2, 0, 0, q, idx, 0.5)
    vf2 = W.bf16_bits_to_f32(v2[0, 0, idx]).astype(np.float64)
    assert np.all(out2 <= vf2.max(axis=0) + 1e-12) and np.all(out2 >= vf2.min(axis=0) - 1e-12)


def test_permutation_invariance_and_two_token_closed_form():
    rng = np.random.default_rng(14)
    cache, k, v = make_cache(rng, 1, 1, 100)
    q = W.f32_to_bf16_bits(rng.standard_normal(128, dtype=np.float32))
    idx = np.sort(rng.choice(100, 20, replace=False)).astype(np.int32)
    a = oracle.gather_attend(cache, 0, 0, q, idx, 0.2)
    b = oracle.gather_attend(cache, 0, 0, q, idx[::-1].copy(), 0.2)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    # two tokens: o = sigmoid(l0 - l1) v0 + sigmoid(l1 - l0) v1
    i, j = 4, 77
    qf = W.bf16_bits_to_f32(q).astype(np.float64)
    kf = W.bf16_bits_to_f32(k[0, 0]).astype(np.float64)
    vf = W.bf16_bits_to_f32(v[0, 0]).astype(np.float64)
    scale = 0.2
    li, lj = scale * qf @ kf[i], scale * qf @ kf[j]
    wi = 1.0 / (1.0 + math.exp(lj - li))
    want = wi * vf[i] + (1.0 - wi) * vf[j]
    got = oracle.gather_attend(cache, 0, 0, q, np.array([i, j], dtype=np.int32), scale)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


def test_large_logits_do_not_overflow():
    """Max-subtracted softmax: logits around +-400 still give finite, correct weights."""
    rng = np.random.default_rng(15)
    cache, k, v = make_cache(rng, 1, 1, 16, scale=30.0)
    q = W.f32_to_bf16_bits(rng.standard_normal(128, dtype=np.float32) * 3)
    idx = np.arange(16, dtype=np.int32)
    out = oracle.gather_attend(cache, 0, 0, q, idx, 1.0)
    assert np.all(np.isfinite(out))
    qf = W.bf16_bits_to_f32(q).astype(np.float64)
    logits = W.bf16_bits_to_f32(k[0, 0]).astype(np.float64) @ qf
    assert np.abs(logits).max() > 100
    w = torch.softmax(torch.from_numpy(logits), dim=0).numpy()
    np.testing.assert_allclose(out, w @ W.bf16_bits_to_f32(v[0, 0]).astype(np.float64),
                               rtol=1e-10, atol=1e-12)


def test_gqa_head_and_batch_addressing():
    """Rows are taken from the named (sequence, KV head), not another one."""
    rng = np.random.default_rng(16)
    cache, k, v = make_cache(rng, 3, 4, 33)
    q = W.f32_to_bf16_bits(rng.standard_normal(128, dtype=np.float32))
    for b, h, t in [(0, 0, 0), (2, 3, 32), (1, 2, 5)]:
        out = oracle.gather_attend(cache, b, h, q, np.array([t], dtype=np.int32), 1.0)
        np.testing.assert_array_equal(out, W.bf16_bits_to_f32(v[b, h, t]).astype(np.float64))


def test_paged_layout_equals_contiguous():
    rng = np.random.default_rng(17)
    B, H, N, d, ps = 2, 2, 70, 128, 16
    cache, k, v = make_cache(rng, B, H, N)
    pages_per = (N + ps - 1) // ps
    perm = rng.permutation(B * pages_per).astype(np.int32)
    table = perm.reshape(B, pages_per).copy()
    kp = np.zeros((B * pages_per, H, ps, d), dtype=np.uint16)
    vp = np.zeros_like(kp)
    for b in range(B):
        for t in range(N):
            kp[table[b, t // ps], :, t % ps] = k[b, :, t]
            vp[table[b, t // ps], :, t % ps] = v[b, :, t]
    pc = oracle.Cache(kp, vp, np.zeros(kp.shape[:3], np.uint32), np.full(B, N, np.int32),
                      page_table=table, page_size=ps)
    q = W.f32_to_bf16_bits(rng.standard_normal(128, dtype=np.float32))
    idx = np.sort(rng.choice(N, 25, replace=False)).astype(np.int32)
    for b in range(B):
        for h in range(H):
            a = oracle.gather_attend(cache, b, h, q, idx, 0.09)
            c = oracle.gather_attend(pc, b, h, q, idx, 0.09)
            np.testing.assert_array_equal(a, c)


def test_empty_index_set_gives_zeros():
    rng = np.random.default_rng(18)
    cache, _, _ = make_cache(rng, 1, 1, 8)
    q = W.f32_to_bf16_bits(rng.standard_normal(128, dtype=np.float32))
    out = oracle.gather_attend(cache, 0, 0, q, np.zeros(0, dtype=np.int32), 1.0)
    assert np.all(out == 0.0)
