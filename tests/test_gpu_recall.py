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


@pytest.mark.parametrize("mapping,window", [("shared-projection", (0, 0)), ("independent-mlp", (0, 0)),
                                            ("shared-projection", (128, 128))])
def test_recall_equals_the_all_oracle_recall_on_the_oracle_codes(mapping, window):
    """On codes computed by the oracle, the index sets of the HIP path are the oracle's, so the recall the
    harness reports is exactly the one obtained with no GPU in the loop (not merely above a threshold)."""
    _, per_head, per_head_oracle = rh.measure(8192, sparsity=16, k_true=32, mapping=mapping, n_sink=window[0],
                                              n_local=window[1], oracle_codes=True)
    assert per_head == per_head_oracle
    assert len(per_head) == 32
