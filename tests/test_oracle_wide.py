"""Pins for the oracle's wider signatures (b = 32 x words bits per code; the paper's bit-width ablation
and its SCORE latency table use 64 to 512 bits): bit-by-bit counts and hand-built networks written
here, the 32-bit functions as the words = 1 special case, and the whole step as a composition."""
import math

import numpy as np
import pytest

import oracle
import workloads as W


def bit(code_words, j):
    return (int(code_words[j // 32]) >> (j % 32)) & 1


@pytest.mark.parametrize("words", [1, 2, 4, 8, 16])
def test_score_wide_is_bit_by_bit_agreement_count(words):
    rng = np.random.default_rng(words)
    for _ in range(200):
        q = rng.integers(0, 2 ** 32, size=words, dtype=np.uint64).astype(np.uint32)
        k = rng.integers(0, 2 ** 32, size=words, dtype=np.uint64).astype(np.uint32)
        agree = sum(bit(q, j) == bit(k, j) for j in range(32 * words))
        assert oracle.score_wide(q, k) == agree
    assert oracle.score_wide(q, q) == 32 * words
    assert oracle.score_wide(q, ~q) == 0
    if words == 1:
        assert oracle.score_wide(q, k) == oracle.score(int(q[0]), int(k[0]))


def test_score_wide_law_of_uniform_codes():
    rng = np.random.default_rng(9)
    words = 4
    q = rng.integers(0, 2 ** 32, size=words, dtype=np.uint64).astype(np.uint32)
    ks = rng.integers(0, 2 ** 32, size=(20000, words), dtype=np.uint64).astype(np.uint32)
    sc = oracle.scores_wide(q, ks)
    assert all(int(sc[i]) == oracle.score_wide(q, ks[i]) for i in range(0, 20000, 997))
    assert abs(sc.mean() - 64.0) < 0.2 and abs(sc.var() - 32.0) < 1.5        # Binomial(128, 1/2)


@pytest.mark.parametrize("words", [2, 8])
def test_encode_vec_wide_unit_to_bit_order_and_strict_sign(words):
    """One layer that copies input i to unit perm[i] (b <= 128 inputs are enough for b = 64; for wider
    codes units reuse inputs): bit j % 32 of word j / 32 is the sign of the copied input."""
    b = 32 * words
    rng = np.random.default_rng(3)
    src = rng.integers(0, 128, size=b)                      # unit j reads input src[j]
    Wm = np.zeros((1, 128, b), dtype=np.float32)
    Wm[0, src, np.arange(b)] = 1.0
    x = rng.standard_normal(128).astype(np.float32)
    x[src[5]] = 0.0                                         # sign(0) -> bit 0
    xb = W.f32_to_bf16_bits(x)
    code, act = oracle.encode_vec_wide(oracle.Mlp([Wm]), 0, xb, words)
    xf = W.bf16_bits_to_f32(xb)
    for j in range(b):
        assert act[j] == float(xf[src[j]])
        assert bit(code, j) == int(xf[src[j]] > 0)
    assert bit(code, 5) == 0 or xf[src[5]] > 0


def test_encode_vec_wide_words_1_is_the_32_bit_function_and_matches_matmul():
    rng = np.random.default_rng(4)
    w32 = W.mapping_weights(rng, 2, (128, 128, 32))
    x = W.f32_to_bf16_bits(rng.standard_normal(128).astype(np.float32))
    c1, a1 = oracle.encode_vec(oracle.Mlp(w32), 1, x)
    cw, aw = oracle.encode_vec_wide(oracle.Mlp(w32), 1, x, 1)
    assert int(cw[0]) == int(c1) and np.array_equal(a1, aw)
    w256 = W.mapping_weights(rng, 2, (128, 64, 256))
    cw, aw = oracle.encode_vec_wide(oracle.Mlp(w256), 1, x, 8)
    xf = W.bf16_bits_to_f32(x).astype(np.float64)
    h = xf @ w256[0][1].astype(np.float64)
    h = h / (1.0 + np.exp(-h))
    z = h @ w256[1][1].astype(np.float64)
    np.testing.assert_allclose(aw, z, rtol=1e-12, atol=1e-13)
    for j in range(256):
        assert bit(cw, j) == int(z[j] > 0)


def test_decode_step_wide_is_the_composition_of_its_parts():
    words = 4
    cfg = W.scaled(W.c1(context=300, k=20, batch=2), name="wide", mlp_dims=(128, 128, 32 * words))
    L = W.make_layer(cfg, 5)
    L.seq_lens[1] = 111
    g = cfg.group
    phi_q, phi_kv = oracle.Mlp(L.w_q), oracle.Mlp(L.w_kv)
    cache = oracle.Cache(L.k, L.v, np.zeros(L.k.shape[:3], dtype=np.uint32), L.seq_lens.copy())
    codes = np.zeros(L.k.shape[:3] + (words,), dtype=np.uint32)
    oracle.encode_keys_wide(phi_kv, cache, codes, None, None, 300)
    assert not codes[1, :, 111:].any() and codes[1, :, :111].any()
    scale = 1.0 / math.sqrt(128)
    res = oracle.decode_step_wide(phi_q, phi_kv, cache, codes, L.q, L.k_per_seq, scale, n_sink=3, n_local=4)
    qc, _ = oracle.encode_query_wide(phi_q, L.q, words)
    assert np.array_equal(qc, res["q_codes"])
    for b in range(2):
        n = int(L.seq_lens[b])
        for h in (0, 9, 31):
            kc, _ = oracle.encode_vec_wide(phi_kv, h // g, L.k[b, h // g, 7], words)
            assert np.array_equal(kc, codes[b, h // g, 7])
            sc = oracle.scores_wide(qc[b, h], codes[b, h // g, :n])
            want, thr, got = oracle.topk_window(sc, 20, 3, 4)
            cnt = int(res["count"][b, h])
            assert res["idx"][b, h, :cnt].tolist() == want.tolist() and res["threshold"][b, h] == thr
            o = oracle.gather_attend(cache, b, h // g, L.q[b, h], want, scale)
            np.testing.assert_allclose(res["out"][b, h], o, rtol=0, atol=1e-14)
