"""Which differences between two runs of the PSD decisions can be blamed on near-ties.

The decision kernels are bit-exact given the same (top1, conf) tables.  A bf16 model call, however, returns
confidences that differ from the oracle's by a relative error of up to r (a logit error of eps moves a softmax
probability by at most a factor exp(2 eps)), and ranking / thresholding are discontinuous: two positions whose
oracle confidences lie within a factor (1 + r)^2 of each other may legitimately come out in the other order, and a
confidence within a factor (1 + r) of tau on the other side of it.  Nothing else may differ.  The functions here
name the pairs (or the threshold crossings) that actually differ between the two sides and say which of them are
NOT covered by such a near-tie; the tests assert that none is.  Host-side test logic only (no model arithmetic).
"""
from typing import List, Sequence, Tuple

import numpy as np


def near_pair(o_conf: np.ndarray, i: int, j: int, r: float) -> bool:
    """Oracle confidences of positions i and j within a factor (1 + r)^2 of each other."""
    a, b = float(o_conf[i]), float(o_conf[j])
    if a <= 0 or b <= 0:
        return False
    return max(a, b) <= min(a, b) * (1.0 + r) ** 2


def near_tau(o_conf: np.ndarray, i: int, tau: float, r: float) -> bool:
    c = float(o_conf[i])
    return np.isfinite(tau) and c > 0 and tau / (1.0 + r) <= c <= tau * (1.0 + r)


def unexplained_commit_differences(o_conf: np.ndarray, T_o: Sequence[int], T_g: Sequence[int], tau: float,
                                   r: float) -> List[Tuple[str, int]]:
    """T_o / T_g: block positions the policy commits on the oracle's / the other side's tables.  A position in one set
    only is explained by a threshold crossing next to tau, or by a position of the other set-difference that swapped
    rank with it (a near pair).  Returns the positions left unexplained."""
    only_o, only_g = sorted(set(T_o) - set(T_g)), sorted(set(T_g) - set(T_o))
    bad = []
    for i, others, tag in [(i, only_g, "oracle-only") for i in only_o] + [(i, only_o, "other-only") for i in only_g]:
        if near_tau(o_conf, i, tau, r) or any(near_pair(o_conf, i, j, r) for j in others):
            continue
        bad.append((tag, int(i)))
    return bad


def inverted_pairs(order_o: Sequence[int], order_g: Sequence[int], n_ranks: int) -> List[Tuple[int, int]]:
    """Pairs (i, j) of positions among the first n_ranks of either ordering whose relative order differs between the
    two orderings (a position missing from an ordering counts as ranked behind all present ones)."""
    pos_o = {p: k for k, p in enumerate(order_o)}
    pos_g = {p: k for k, p in enumerate(order_g)}
    live = sorted(set(list(order_o[:n_ranks]) + list(order_g[:n_ranks])))
    big = len(order_o) + len(order_g) + 1
    out = []
    for a in range(len(live)):
        for b in range(a + 1, len(live)):
            i, j = live[a], live[b]
            so = pos_o.get(i, big) - pos_o.get(j, big)
            sg = pos_g.get(i, big) - pos_g.get(j, big)
            if so * sg < 0 or (so == 0) != (sg == 0):
                out.append((int(i), int(j)))
    return out


def unexplained_rank_differences(o_conf: np.ndarray, sigma_o: Sequence[int], sigma_g: Sequence[int], n_ranks: int,
                                 r: float) -> List[Tuple[int, int]]:
    """sigma_o / sigma_g: the speculative orderings (block positions, most confident first) from the oracle's and the
    other side's tables over the SAME residual set.  Only the first n_ranks feed the drafts.  Returns the inverted
    pairs that are not near pairs."""
    return [(i, j) for i, j in inverted_pairs(list(sigma_o), list(sigma_g), n_ranks) if not near_pair(o_conf, i, j, r)]


def edge_verdicts(v_top1: np.ndarray, drafted: np.ndarray, positions: Sequence[int], committed_by_policy) -> np.ndarray:
    """verdict[p, a] for parent node p and speculated position positions[a]: parent p's verifier predicts the drafted
    token drafted[j] there AND the policy applied to p's verifier output commits it (the per-position test of the
    acceptance criterion; committed_by_policy(p) -> set of block positions)."""
    K = v_top1.shape[0]
    out = np.zeros((K, len(positions)), dtype=bool)
    for p in range(K):
        T_p = committed_by_policy(p)
        for a, j in enumerate(positions):
            out[p, a] = int(v_top1[p, j]) == int(drafted[j]) and j in T_p
    return out
