"""Pins for the oracle's SCORE (section 4.1, eq. 1) and TOPK (section 4).

The oracle is checked against things other than itself: a bit-by-bit count
written here, algebraic identities of the Hamming similarity, the binomial law
of uniform codes, and an exhaustive search over subsets for tiny inputs.
"""
import itertools
import math

import numpy as np
import pytest

import oracle
import workloads as W


def bits_differing(a: int, b: int) -> int:
    n = 0
    for j in range(32):
        n += ((a >> j) & 1) != ((b >> j) & 1)
    return n


def test_score_equals_bit_by_bit_count():
    rng = np.random.default_rng(1)
    pairs = rng.integers(0, 2 ** 32, size=(2000, 2), dtype=np.uint64)
    for a, b in pairs:
        assert oracle.score(int(a), int(b)) == 32 - bits_differing(int(a), int(b))


def test_score_identities():
    rng = np.random.default_rng(2)
    xs = rng.integers(0, 2 ** 32, size=200, dtype=np.uint64)
    for x in xs:
        x = int(x)
        assert oracle.score(x, x) == 32
        assert oracle.score(x, x ^ 0xFFFFFFFF) == 0
        y = int(rng.integers(0, 2 ** 32, dtype=np.uint64))
        assert oracle.score(x, y) == oracle.score(y, x)
        # flipping one more differing bit lowers the similarity by exactly one
        j = int(rng.integers(0, 32))
        assert abs(oracle.score(x, y) - oracle.score(x, y ^ (1 << j))) == 1
    for j in range(32):
        assert oracle.score(0, 1 << j) == 31
        assert oracle.score(0xFFFFFFFF, 1 << j) == 1
    assert oracle.score(0, 0x80000000) == 31          # top bit is counted (no sign trouble)


def test_scores_vector_matches_scalar_and_binomial_law():
    L = W.make_layer(W.c0())
    qc = int(L.q_codes[0, 0])
    kc = L.k_codes[0, 0]
    sc = oracle.scores(qc, kc)
    for i in range(0, kc.shape[0], 97):
        assert sc[i] == 32 - bits_differing(qc, int(kc[i]))
    # uniform codes: similarity ~ Binomial(32, 1/2); mean 16, variance 8
    n = sc.shape[0]
    assert abs(sc.mean() - 16.0) < 5 * math.sqrt(8.0 / n)
    assert abs(sc.var() - 8.0) < 0.6
    p_ge_21 = sum(math.comb(32, s) for s in range(21, 33)) / 2 ** 32
    assert abs((sc >= 21).mean() - p_ge_21) < 5 * math.sqrt(p_ge_21 / n)


# ---------------------------------------------------------------- TOPK
def brute_force_topk(scores, k):
    """Search all size-k subsets: valid top-k sets have min(selected) >= max(rest); the tie rule
    (lower index wins) picks the lexicographically smallest ascending index tuple among them."""
    n = len(scores)
    ke = min(k, n)
    best = None
    for sub in itertools.combinations(range(n), ke):   # generated in lexicographic order
        rest = [scores[i] for i in range(n) if i not in sub]
        if not rest or min(scores[i] for i in sub) >= max(rest):
            best = sub
            break
    return list(best)


def test_topk_exhaustive_tiny():
    for n in range(1, 8):
        for sc in itertools.product((0, 1, 2), repeat=n):
            arr = np.array(sc, dtype=np.int32)
            for k in range(1, n + 2):
                want = brute_force_topk(sc, k)
                got_s, thr_s = oracle.topk_sort(arr, k)
                got_h, thr_h = oracle.topk_hist(arr, k)
                assert got_s.tolist() == want, (sc, k)
                assert got_h.tolist() == want, (sc, k)
                assert thr_s == thr_h == min(sc[i] for i in want)


@pytest.mark.parametrize("n,k,spread", [(1000, 31, 33), (4096, 256, 33), (5000, 5000, 5),
                                        (3000, 2999, 2), (777, 1, 33), (64, 100, 33)])
def test_topk_sort_equals_hist_and_invariants(n, k, spread):
    rng = np.random.default_rng(n * 131 + k)
    sc = rng.integers(0, spread, size=n).astype(np.int32)
    a, ta = oracle.topk_sort(sc, k)
    b, tb = oracle.topk_hist(sc, k)
    assert a.tolist() == b.tolist() and ta == tb
    ke = min(k, n)
    assert len(a) == ke
    assert np.all(np.diff(a) > 0)                                  # ascending, unique
    sel = np.zeros(n, bool)
    sel[a] = True
    if ke < n:
        assert sc[sel].min() >= sc[~sel].max()
    T = ta
    assert (sc > T).sum() < ke <= (sc >= T).sum()                  # C(T+1) < k <= C(T)
    assert sel[sc > T].all()
    tie = np.flatnonzero(sc == T)
    taken = sel[tie]
    r = ke - int((sc > T).sum())
    assert taken[:r].all() and not taken[r:].any()                 # lowest indices of the tie bucket


def test_topk_all_equal_scores_takes_prefix():
    sc = np.full(100, 17, dtype=np.int32)
    a, t = oracle.topk_sort(sc, 10)
    assert a.tolist() == list(range(10)) and t == 17
    b, _ = oracle.topk_hist(sc, 10)
    assert b.tolist() == list(range(10))


def test_c0_threshold_matches_binomial_tail():
    """Uniform codes, 16x sparsity: P[s>=21] = 5.5 % < 6.25 % <= P[s>=20] = 10.8 % so T = 20."""
    p = lambda s0: sum(math.comb(32, s) for s in range(s0, 33)) / 2 ** 32
    assert p(21) < 1 / 16 <= p(20)
    assert p(22) < 1 / 32 <= p(21)
    L = W.make_layer(W.c0())
    sc = oracle.scores(int(L.q_codes[0, 0]), L.k_codes[0, 0])
    _, T = oracle.topk_sort(sc, 256)
    assert T == 20
