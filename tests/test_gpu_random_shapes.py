"""Seeded random shapes for SCORE + TOPK (with and without the kept window) + GATHER-ATT through the C ABI:
lengths (empty and one-token sequences included), budgets (zero and larger than the sequence included), group
sizes, kept windows longer than the sequence, and code distributions with few distinct scores.  Every (sequence,
head) is compared with the oracle: ids, counts and thresholds bit-exact, outputs within the tolerance."""
import numpy as np
import pytest

from test_gpu_window import window_case

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("topk_path")]


def draw_case(rng):
    tier = rng.integers(0, 3)
    n = int((rng.integers(1, 300), rng.integers(1000, 6000), rng.integers(20000, 70000))[tier])
    batch = int(rng.integers(1, 5))
    hkv = int(rng.choice([1, 2]))
    group = int(rng.choice([1, 2, 4, 8]))
    lens = [int(x) for x in rng.integers(0, n + 1, size=batch)]
    lens[int(rng.integers(0, batch))] = n                             # one sequence has the full length
    if rng.random() < 0.3:
        lens[int(rng.integers(0, batch))] = int(rng.choice([0, 1]))
    k = int(rng.integers(1, max(2, n // 4)))
    k_per_seq = None
    if rng.random() < 0.5:
        k_per_seq = [int(x) for x in rng.integers(0, k + 1, size=batch)]
        k_per_seq[int(rng.integers(0, batch))] = k
    n_sink, n_local = (0, 0) if rng.random() < 0.3 else (int(rng.integers(0, 200)), int(rng.integers(0, 200)))
    kind = int(rng.integers(0, 3))
    return dict(n=n, batch=batch, hkv=hkv, group=group, lens=lens, k=k, k_per_seq=k_per_seq, n_sink=n_sink,
                n_local=n_local, kind=kind)


def codes_of(kind, rng):
    if kind == 0:                                                      # uniform codes
        return lambda s: rng.integers(0, 2 ** 32, size=s, dtype=np.uint64).astype(np.uint32)
    if kind == 1:                                                      # three distinct codes: long runs of ties
        pool = rng.integers(0, 2 ** 32, size=3, dtype=np.uint64).astype(np.uint32)
        return lambda s: pool[rng.integers(0, 3, size=s)]
    return lambda s: (rng.integers(0, 2 ** 32, size=s, dtype=np.uint64).astype(np.uint32) & np.uint32(0x0000FFFF))  # scores in a narrow band


@pytest.mark.parametrize("chunk", range(6))
def test_random_shapes(chunk):
    rng = np.random.default_rng(977 + chunk)
    for i in range(10):
        c = draw_case(rng)
        print(f"case {chunk}.{i}: {c}", flush=True)
        window_case(c["n"], c["k"], c["n_sink"], c["n_local"], codes_of(c["kind"], rng), batch=c["batch"],
                    Hq=c["hkv"] * c["group"], Hkv=c["hkv"], lens=c["lens"], k_per_seq=c["k_per_seq"],
                    check_out=c["n"] < 6000)


@pytest.mark.parametrize("seed", range(5))
def test_random_paged_whole_steps(seed):
    """Paged caches with random page tables, mixed lengths and a budget per sequence: the whole step
    (key codes, query codes, SCORE + TOPK, GATHER-ATT), staged against the oracle."""
    import workloads as W
    import gpu_util
    import test_gpu_parity
    test_gpu_parity.gu = gpu_util                      # that module binds it in a fixture of its own
    run_whole_step = test_gpu_parity.run_whole_step
    rng = np.random.default_rng(4242 + seed)
    lo = int(rng.integers(1, 400))
    hi = int(rng.integers(lo + 16, 9000))
    batch = int(rng.integers(1, 7))
    heads = [(32, 8), (8, 8), (16, 2), (8, 1)][int(rng.integers(0, 4))]
    cfg = W.scaled(W.c4(batch=batch, lo=lo, hi=hi), planted=int(rng.integers(0, 6)), n_q_heads=heads[0],
                   n_kv_heads=heads[1], k_divisor=int(rng.choice([4, 16, 32])))
    print(f"paged case {seed}: batch={batch} lengths in [{lo}, {hi}] heads={heads} k=N/{cfg.k_divisor}", flush=True)
    L = W.make_layer(cfg, seed=500 + seed)
    run_whole_step(L)


@pytest.mark.parametrize("heads", [(6, 3), (5, 5), (12, 6), (4, 4)])
def test_paged_head_counts_odd_and_even(heads):
    """Paged SCORE + TOPK numbers its workgroups so that neighbouring KV heads share a cache line's fetch, with
    a plain order for an odd head count: whole steps at both kinds, more items than one group of eight."""
    import workloads as W
    import gpu_util
    import test_gpu_parity
    test_gpu_parity.gu = gpu_util
    cfg = W.scaled(W.c4(batch=5, lo=40, hi=9000), planted=4, n_q_heads=heads[0], n_kv_heads=heads[1], k_divisor=16)
    L = W.make_layer(cfg, seed=900 + heads[0])
    test_gpu_parity.run_whole_step(L)
