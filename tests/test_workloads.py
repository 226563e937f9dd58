"""Host-side checks of the synthetic input generator and of the byte accounting."""
import os

import numpy as np

import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "kv_cache_sizing.txt")


def golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_kv_sizing_matches_the_papers_figures():
    (layers, hkv, d, elt, mib_per_token, tokens, gib_total), (bits,) = golden_rows()
    per_token = W.kv_cache_bytes_per_token(int(layers), int(hkv), int(d))
    assert int(elt) == 2
    assert per_token == float(mib_per_token) * 2 ** 20
    assert per_token * int(tokens) == int(gib_total) * 2 ** 30
    assert W.BITS == int(bits)


def test_algorithmic_bytes_formula():
    # per sequence: 32 N + 16384 k + 16384 bytes for the Llama shape
    for n, k in ((32768, 1024), (131072, 4096), (524288, 16384)):
        assert W.algorithmic_bytes(8, 32, 128, [n], [k]) == 32 * n + 16384 * k + 16384
    assert W.algorithmic_bytes(8, 32, 128, [100, 100], [200, 10]) == \
        2 * (32 * 100 + 16384) + 16384 * (100 + 10)


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.140625], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    got = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x))
    np.testing.assert_array_equal(got, np.array([1.0, 1.0, 1.015625, -2.5, 0.0, 3.140625], np.float32))


def test_generator_is_deterministic_and_shaped():
    cfg = W.scaled(W.c1(), context=512, k=16, planted=8)
    a, b = W.make_layer(cfg), W.make_layer(cfg)
    for name in ("q", "k", "v", "seq_lens", "k_per_seq", "planted_pos"):
        np.testing.assert_array_equal(getattr(a, name), getattr(b, name))
    assert a.k.shape == (1, 8, 512, 128) and a.q.shape == (1, 32, 128)
    assert [w.shape for w in a.w_q] == [(32, 128, 128), (32, 128, 32)]
    assert [w.shape for w in a.w_kv] == [(8, 128, 128), (8, 128, 32)]
    # planted positions are disjoint inside a KV head
    for hk in range(8):
        pos = a.planted_pos[0, hk * 4:(hk + 1) * 4].ravel()
        assert len(set(pos.tolist())) == len(pos)


def test_paged_mixed_batch_layout():
    cfg = W.scaled(W.c4(batch=5, lo=40, hi=300), planted=2)
    L = W.make_layer(cfg)
    assert L.page_table is not None and L.k.shape[2] == 16
    assert np.all((L.seq_lens >= 40) & (L.seq_lens <= 300))
    np.testing.assert_array_equal(L.k_per_seq, (L.seq_lens + 15) // 16)
    used = L.page_table[L.page_table >= 0]
    assert len(set(used.tolist())) == len(used) == L.k.shape[0]      # a permutation of the pool
    for b in range(5):
        n_pages = (int(L.seq_lens[b]) + 15) // 16
        assert np.all(L.page_table[b, :n_pages] >= 0) and np.all(L.page_table[b, n_pages:] == -1)
