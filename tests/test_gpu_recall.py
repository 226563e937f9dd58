"""The synthetic recall harness on the GPU path (sections 4 and 4.2; the paper's recall figure uses the
top-32 tokens at 16x sparsity): a mapping that hashes the angle recalls the planted pivotal tokens,
unrelated query/key mappings stay near chance, and the always-kept window only adds tokens."""
import pytest

import recall_harness as rh

pytestmark = pytest.mark.gpu


def test_shared_projection_recalls_planted_tokens():
    r, per_head = rh.measure(8192, sparsity=16, k_true=32, mapping="shared-projection")
    assert r >= 0.95, per_head
    r32, _ = rh.measure(8192, sparsity=32, k_true=32, mapping="shared-projection", heads=range(0, 32, 4))
    assert r32 >= 0.9


def test_independent_mappings_stay_near_chance():
    r, per_head = rh.measure(8192, sparsity=16, k_true=32, mapping="independent-mlp")
    assert r <= 0.25, per_head           # chance is 1/16


def test_window_never_lowers_recall():
    heads = range(0, 32, 8)
    base, _ = rh.measure(4096, sparsity=64, k_true=32, mapping="independent-mlp", heads=heads)
    win, _ = rh.measure(4096, sparsity=64, k_true=32, mapping="independent-mlp", heads=heads, n_sink=128, n_local=128)
    assert win >= base
