"""Pins for the oracle's mapping phi (section 4.1, eq. 2), the key-code store and the
composed decode step.

Pins: hand-built networks with known outputs (bit order, strict sign, SiLU, bias,
operand orientation), the random-signed-projection law P[bit differs] = theta/pi
that section 4.3 refers to, complement symmetry of bias-free linear maps, and a
matmul library route in float64.
"""
import math

import numpy as np
import pytest

import oracle
import workloads as W


def bf(x):
    return W.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def silu(z):
    return z / (1.0 + math.exp(-z))


def test_bit_order_and_strict_sign():
    d = 128
    Wm = np.zeros((1, d, 32), dtype=np.float32)
    for j in range(32):
        Wm[0, j, j] = 1.0                      # output unit j = x_j
    mlp = oracle.Mlp([Wm])
    for j in (0, 1, 5, 31):
        x = np.full(d, -1.0, dtype=np.float32)
        x[j] = 2.0
        code, act = oracle.encode_vec(mlp, 0, bf(x))
        assert int(code) == (1 << j)           # unit j -> bit j, LSB = unit 0
        assert act[j] == 2.0 and act[(j + 1) % 32] == -1.0
    x = np.zeros(d, dtype=np.float32)          # sign(0) = 0 -> bit 0
    code, act = oracle.encode_vec(mlp, 0, bf(x))
    assert int(code) == 0 and np.all(act == 0.0)
    x[:32] = 1.0
    assert int(oracle.encode_vec(mlp, 0, bf(x))[0]) == 0xFFFFFFFF


def test_operand_orientation_non_square():
    """y = x W with W [in, out]: a transposed read of a non-square matrix gives other bits."""
    d = 128
    rng = np.random.default_rng(20)
    Wm = rng.standard_normal((2, d, 32)).astype(np.float32)
    x = bf(rng.standard_normal(d, dtype=np.float32))
    xf = W.bf16_bits_to_f32(x).astype(np.float64)
    for h in range(2):
        code, act = oracle.encode_vec(oracle.Mlp([Wm]), h, x)
        want = xf @ Wm[h].astype(np.float64)
        np.testing.assert_allclose(act, want, rtol=1e-12, atol=1e-12)
        bits = sum((1 << j) for j in range(32) if want[j] > 0)
        assert int(code) == bits


def test_silu_between_layers_and_bias_closed_form():
    d = 128
    W1 = np.zeros((1, d, d), dtype=np.float32)
    W1[0, 0, 0] = 1.0
    W1[0, 1, 1] = 1.0
    W2 = np.zeros((1, d, 32), dtype=np.float32)
    W2[0, 0, 0] = 1.0      # a0 = silu(z0)
    W2[0, 1, 1] = 1.0      # a1 = silu(z1) + 0.1
    W2[0, 0, 2] = 1.0      # a2 = silu(z0) + silu(z1)
    W2[0, 1, 2] = 1.0
    b2 = np.zeros((1, 32), dtype=np.float32)
    b2[0, 1] = 0.1
    b2[0, 3] = -0.5        # a3 = -0.5 (bias only)
    b2[0, 4] = 0.25        # a4 = +0.25
    mlp = oracle.Mlp([W1, W2], [None, b2])
    x = np.zeros(d, dtype=np.float32)
    x[0], x[1] = 2.0, -2.0
    code, act = oracle.encode_vec(mlp, 0, bf(x))
    np.testing.assert_allclose(act[0], silu(2.0), rtol=1e-14)
    np.testing.assert_allclose(act[1], silu(-2.0) + np.float64(np.float32(0.1)), rtol=1e-14)
    np.testing.assert_allclose(act[2], silu(2.0) + silu(-2.0), rtol=1e-14)
    assert act[3] == -0.5 and act[4] == 0.25
    # silu(-2)+0.1 < 0 (a ReLU would give +0.1); silu(2)+silu(-2) > 0 (no activation would give 0)
    assert int(code) == (1 << 0) | (1 << 2) | (1 << 4)


def test_three_layer_network_matches_float64_matmul():
    rng = np.random.default_rng(21)
    ws = W.mapping_weights(rng, 3, (128, 128, 128, 32))
    bs = [rng.uniform(-0.1, 0.1, size=(3, w.shape[2])).astype(np.float32) for w in ws]
    mlp = oracle.Mlp(ws, bs)
    q = bf(rng.standard_normal((4, 3, 128), dtype=np.float32))
    codes, act = oracle.encode_query(mlp, q)
    xf = W.bf16_bits_to_f32(q).astype(np.float64)
    for b in range(4):
        for h in range(3):
            z = xf[b, h]
            for l in range(3):
                z = z @ ws[l][h].astype(np.float64) + bs[l][h].astype(np.float64)
                if l < 2:
                    z = z / (1.0 + np.exp(-z))
            np.testing.assert_allclose(act[b, h], z, rtol=1e-11, atol=1e-13)
            assert int(codes[b, h]) == sum((1 << j) for j in range(32) if z[j] > 0)


def test_linear_map_complement_symmetry():
    rng = np.random.default_rng(22)
    Wm = rng.standard_normal((1, 128, 32)).astype(np.float32)
    mlp = oracle.Mlp([Wm])
    for _ in range(20):
        x = rng.standard_normal(128, dtype=np.float32)
        c1, _ = oracle.encode_vec(mlp, 0, bf(x))
        c2, _ = oracle.encode_vec(mlp, 0, bf(-x))
        assert int(c1) ^ int(c2) == 0xFFFFFFFF


def test_random_signed_projections_follow_theta_over_pi():
    """One linear layer with a shared Gaussian W is sign-random-projection hashing:
    P[bit differs] = theta / pi for two vectors at angle theta."""
    rng = np.random.default_rng(23)
    d, trials = 128, 400
    for theta in (math.pi / 6, math.pi / 2, 2.2):
        differing = 0
        for t in range(trials):
            Wm = rng.standard_normal((1, d, 32)).astype(np.float32)
            mlp = oracle.Mlp([Wm])
            u = rng.standard_normal(d)
            u /= np.linalg.norm(u)
            w = rng.standard_normal(d)
            w -= (w @ u) * u
            w /= np.linalg.norm(w)
            x = 8.0 * u
            y = 8.0 * (math.cos(theta) * u + math.sin(theta) * w)
            cx, _ = oracle.encode_vec(mlp, 0, bf(x))
            cy, _ = oracle.encode_vec(mlp, 0, bf(y))
            differing += 32 - oracle.score(int(cx), int(cy))
        n_bits = 32 * trials
        p = theta / math.pi
        assert abs(differing / n_bits - p) < 5 * math.sqrt(p * (1 - p) / n_bits) + 2e-3


# ------------------------------------------------------------ key-code store
def small_layer(**kw):
    cfg = W.scaled(W.c1(), context=300, k=16, batch=2, planted=4, **kw)
    return W.make_layer(cfg, seed=99)


def test_encode_keys_in_place_and_append():
    L = small_layer()
    B, Hkv, N, d = L.k.shape
    phi = oracle.Mlp(L.w_kv)
    codes = np.zeros((B, Hkv, N), dtype=np.uint32)
    lens = np.array([300, 200], dtype=np.int32)
    cache = oracle.Cache(L.k, L.v, codes, lens)
    act = oracle.encode_keys(phi, cache, None, None, 300, want_act=True)
    assert lens.tolist() == [300, 200]                       # in-place mode leaves lengths alone
    for b, h, t in [(0, 0, 0), (0, 7, 299), (1, 3, 199), (1, 0, 0)]:
        c, a = oracle.encode_vec(phi, h, L.k[b, h, t])
        assert codes[b, h, t] == c
        slot = t - max(0, int(lens[b]) - 300)
        np.testing.assert_array_equal(act[b, h, slot], a)
    assert np.all(codes[1, :, 200:] == 0)                    # rows past seq_len untouched
    # append two tokens to a shorter cache
    lens2 = np.array([100, 50], dtype=np.int32)
    k2, v2, codes2 = L.k.copy(), L.v.copy(), np.zeros_like(codes)
    cache2 = oracle.Cache(k2, v2, codes2, lens2)
    rng = np.random.default_rng(5)
    k_new = bf(rng.standard_normal((B, Hkv, 2, d), dtype=np.float32))
    v_new = bf(rng.standard_normal((B, Hkv, 2, d), dtype=np.float32))
    oracle.encode_keys(phi, cache2, k_new, v_new, 2)
    assert lens2.tolist() == [102, 52]
    for b, pos in ((0, 100), (1, 50)):
        for j in range(2):
            np.testing.assert_array_equal(k2[b, :, pos + j], k_new[b, :, j])
            np.testing.assert_array_equal(v2[b, :, pos + j], v_new[b, :, j])
            for h in (0, 5):
                assert codes2[b, h, pos + j] == oracle.encode_vec(phi, h, k_new[b, h, j])[0]
    np.testing.assert_array_equal(k2[0, :, :100], L.k[0, :, :100])
    assert np.all(codes2[0, :, :100] == 0) and np.all(codes2[0, :, 102:] == 0)


def test_decode_step_is_the_composition_of_its_parts():
    L = small_layer()
    B, Hkv, N, d = L.k.shape
    Hq, g = L.cfg.n_q_heads, L.cfg.group
    phi_q, phi_kv = oracle.Mlp(L.w_q), oracle.Mlp(L.w_kv)
    codes = np.zeros((B, Hkv, N), dtype=np.uint32)
    lens = L.seq_lens.copy()
    cache = oracle.Cache(L.k, L.v, codes, lens)
    oracle.encode_keys(phi_kv, cache, None, None, N)
    scale = 1.0 / math.sqrt(d)
    kps = np.array([16, 9], dtype=np.int32)
    res = oracle.decode_step(phi_q, phi_kv, cache, L.q, kps, scale)
    qc, _ = oracle.encode_query(phi_q, L.q)
    np.testing.assert_array_equal(res["q_codes"], qc)
    for b in range(B):
        for h in range(Hq):
            sc = oracle.scores(int(qc[b, h]), codes[b, h // g, :lens[b]])
            idx, T = oracle.topk_hist(sc, int(kps[b]))
            cnt = res["count"][b, h]
            assert cnt == kps[b] and res["threshold"][b, h] == T
            np.testing.assert_array_equal(res["idx"][b, h, :cnt], idx)
            out = oracle.gather_attend(cache, b, h // g, L.q[b, h], idx, scale)
            np.testing.assert_array_equal(res["out"][b, h], out)


def test_decode_step_append_scores_the_new_token():
    """The appended token takes part in this step's scoring: with k = N every token,
    including the new one at position N-1, is selected and the output is dense SDPA."""
    cfg = W.scaled(W.c2(batch=2, context=65), k=65, planted=2)
    L = W.make_layer(cfg, seed=7)
    B, Hkv, N, d = L.k.shape
    assert N == 65 and L.seq_lens.tolist() == [64, 64]
    phi_q, phi_kv = oracle.Mlp(L.w_q), oracle.Mlp(L.w_kv)
    codes = np.zeros((B, Hkv, N), dtype=np.uint32)
    lens = L.seq_lens.copy()
    cache = oracle.Cache(L.k, L.v, codes, lens)
    oracle.encode_keys(phi_kv, cache, None, None, 64)
    res = oracle.decode_step(phi_q, phi_kv, cache, L.q, L.k_per_seq, 0.1,
                             k_new=L.k_new, v_new=L.v_new)
    assert lens.tolist() == [65, 65]
    assert np.all(res["count"] == 65)
    for b in range(B):
        for h in (0, 13, 31):
            assert res["idx"][b, h].tolist() == list(range(65))
            dense = oracle.dense_attend(cache, b, h // 4, L.q[b, h], 65, 0.1)
            np.testing.assert_allclose(res["out"][b, h], dense, rtol=1e-12, atol=1e-14)
            np.testing.assert_array_equal(L.k[b, h // 4, 64], L.k_new[b, h // 4])


def test_planted_keys_share_codes_under_shared_linear_hash():
    """Recall sanity (section 4, recall definition): with one shared linear sign-projection for
    queries and keys, keys planted along q are retrieved far above the k/N chance rate."""
    cfg = W.scaled(W.c1(), context=2048, k=64, batch=1, planted=16)
    L = W.make_layer(cfg, seed=3)
    rng = np.random.default_rng(4)
    shared = rng.standard_normal((1, 128, 32)).astype(np.float32)
    phi_q = oracle.Mlp([np.repeat(shared, 32, axis=0)])
    phi_kv = oracle.Mlp([np.repeat(shared, 8, axis=0)])
    codes = np.zeros(L.k.shape[:3], dtype=np.uint32)
    cache = oracle.Cache(L.k, L.v, codes, L.seq_lens.copy())
    oracle.encode_keys(phi_kv, cache, None, None, 2048)
    res = oracle.decode_step(phi_q, phi_kv, cache, L.q, L.k_per_seq, 1 / math.sqrt(128))
    hits = total = 0
    for h in range(32):
        sel = set(res["idx"][0, h, :res["count"][0, h]].tolist())
        hits += len(sel & set(L.planted_pos[0, h].tolist()))
        total += 16
    assert hits / total > 0.9          # chance level is 64/2048 = 3 %
