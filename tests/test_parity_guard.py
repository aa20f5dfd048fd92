"""The near-tie guard of the lock-step parity tests must blame only the pairs that actually swapped: a decision that
differs for any other reason has to come out as unexplained.  (CPU; mistakes are planted on the oracle's side.)"""
import numpy as np

from oracle import psd_oracle as orc
from tests import parity_guard as G


def _tables(seed, L=32):
    rng = np.random.default_rng(seed)
    conf = (1e-3 * (1.0 + 0.5 * rng.random(L))).astype(np.float32)       # flat confidences, as with random-init weights
    return conf


def test_a_swap_of_two_close_confidences_is_explained_and_a_far_swap_is_not():
    conf = _tables(1)
    order = orc.confidence_order(range(32), conf)
    close = conf.copy()
    i, j = order[0], order[1]
    close[i], close[j] = conf[j] * 1.01, conf[j]                         # 1 % apart
    o = orc.confidence_order(range(32), close)
    flipped = close.copy()
    flipped[o[1]] = close[o[0]] * 1.005                                  # the other side ranks them the other way round
    g = orc.confidence_order(range(32), flipped)
    assert G.inverted_pairs(o, g, 3) == [tuple(sorted((o[0], o[1])))]
    assert G.unexplained_rank_differences(close, o, g, 3, r=0.02) == []
    assert G.unexplained_commit_differences(close, [o[0]], [g[0]], 0.9, 0.02) == []
    # planted mistake: the other side commits a position whose oracle confidence is 30 % lower -- no near pair
    far = int(order[-1])
    bad = G.unexplained_commit_differences(conf, [order[0]], [far], 0.9, 0.02)
    assert ("oracle-only", order[0]) in bad and ("other-only", far) in bad
    wrong = [far] + [p for p in order if p != far]
    assert G.unexplained_rank_differences(conf, order, wrong, 3, r=0.02)


def test_a_guard_that_looked_at_any_close_pair_would_have_passed_the_planted_mistake():
    """There IS a near pair somewhere in the table (positions 5 and 6), but it is not the pair that differs."""
    conf = np.linspace(2e-3, 1e-3, 32).astype(np.float32)
    conf[6] = conf[5] * np.float32(0.999)
    order = orc.confidence_order(range(32), conf)
    assert G.near_pair(conf, 5, 6, 0.01)
    bad = G.unexplained_commit_differences(conf, [order[0]], [order[20]], 0.9, 0.01)
    assert len(bad) == 2


def test_threshold_crossings_are_explained_only_next_to_tau():
    conf = np.array([0.95, 0.905, 0.5, 0.2], dtype=np.float32)
    # the other side sees 0.905 as 0.899: not committed there
    assert G.unexplained_commit_differences(conf, [0, 1], [0], 0.9, 0.01) == []
    # 0.5 committed on one side only: nowhere near tau, no swap partner
    assert G.unexplained_commit_differences(conf, [0, 1], [0, 1, 2], 0.9, 0.01) == [("other-only", 2)]


def test_edge_verdicts_follow_the_acceptance_criterion():
    L, K = 8, 3
    drafted = np.arange(100, 100 + L)
    v_top1 = np.tile(drafted, (K, 1))
    v_top1[1, 4] = 7                                                     # parent 1 predicts another token at position 4
    verdicts = G.edge_verdicts(v_top1, drafted, [2, 4], lambda p: {2} if p == 0 else {2, 4})
    assert verdicts.tolist() == [[True, False], [True, False], [True, True]]
