"""Pins for the oracle's decision logic: policy, drafting, hierarchical acceptance, the loop.

Each pin is something the paper or plain mathematics fixes, coded here independently of the
oracle's own formulation:
  * App. B.2: greedy decoding commits the single most confident masked position per
    forward; PSD run with that policy must reproduce a plain greedy decoder, token by token
    and in the same commit order;
  * root-only graph (K = 1): PSD is plain parallel decoding with pi;
  * Sec. 3.2 stage 3: a draft agreeing with every verified prediction is accepted at full
    depth; the accepted depth is the deepest consistent one (brute force over all paths
    through the subset lattice on tiny inputs);
  * Eq. 2: structure of the drafts; Eq. 1: only positions in T change;
  * every model invocation commits at least one token, so TPF >= 1.
"""
import hashlib
import itertools

import numpy as np
import pytest

import psd_inputs as inp
from oracle import psd_oracle as orc

INF = float("inf")


# ---------------------------------------------------------------- helpers (independent code)


def pseudo_model(vocab, seed, conf_kind="uniform", sticky=0.0):
    """A deterministic stand-in for the dLLM: (top1, conf) are a hash of the whole sequence
    state, so any change of any token changes every prediction (as bidirectional attention
    does).  ``sticky`` > 0 mixes in a state-independent component so that rankings and
    tokens are partly stable across steps, which is what lets drafts be accepted."""
    mask_id = vocab - 1

    def fn(tokens, block_start, L):
        h = hashlib.sha256(np.asarray(tokens, dtype=np.int32).tobytes() + bytes([seed % 256])).digest()
        rng = np.random.default_rng(int.from_bytes(h[:8], "little"))
        base = np.random.default_rng(seed * 7919 + block_start)
        lo, hi = {"uniform": (0.0, 1.0), "low": (0.0, 0.3)}[conf_kind]
        c_state, c_base = rng.random(L), base.random(L)
        t_state = rng.integers(0, vocab - 1, size=L)
        t_base = base.integers(0, vocab - 1, size=L)
        use_base = rng.random(L) < sticky
        conf = (lo + (hi - lo) * np.where(use_base, c_base, c_state)).astype(np.float32)
        top1 = np.where(use_base, t_base, t_state).astype(np.int32)
        blk = np.asarray(tokens[block_start: block_start + L])
        masked = blk == mask_id
        return np.where(masked, top1, blk).astype(np.int32), np.where(masked, conf, np.float32(-1)).astype(np.float32)

    return fn


class Counting:
    def __init__(self, fn):
        self.fn, self.calls = fn, 0

    def __call__(self, *a):
        self.calls += 1
        return self.fn(*a)


def plain_greedy(confidence_fn, tokens, block_start, L, mask_id):
    """App. B.2 "Greedy Decoding": one forward, reveal the single most confident masked position."""
    x = tokens.copy()
    order = []
    while (x[block_start: block_start + L] == mask_id).any():
        top1, conf = confidence_fn(x, block_start, L)
        best, best_c = -1, -INF
        for j in range(L):
            if x[block_start + j] == mask_id and conf[j] > best_c:
                best, best_c = j, conf[j]
        x[block_start + best] = top1[best]
        order.append(block_start + best)
    return x, order


def plain_parallel(confidence_fn, tokens, block_start, L, mask_id, tau):
    """App. B.2 "Confidence Parallel Decoding": reveal all positions whose confidence exceeds
    tau (the most confident one when none does)."""
    x = tokens.copy()
    calls = 0
    while (x[block_start: block_start + L] == mask_id).any():
        top1, conf = confidence_fn(x, block_start, L)
        calls += 1
        live = [j for j in range(L) if x[block_start + j] == mask_id]
        take = [j for j in live if conf[j] > tau]
        if not take:
            take = [max(live, key=lambda j: (conf[j], -j))]
        for j in take:
            x[block_start + j] = top1[j]
    return x, calls


def counting_rank(conf, live, i):
    """Rank of i among live positions by (confidence desc, index asc), by counting."""
    return sum(1 for j in live if conf[j] > conf[i] or (conf[j] == conf[i] and j < i))


def commits_by_definition(conf, live, i, policy):
    r = counting_rank(conf, live, i)
    ok = conf[i] > policy.tau or r < policy.k_min
    return ok and (policy.k_max == 0 or r < policy.k_max)


def brute_force_accept(drafts, block_start, L, S, policy, v_top1, v_conf, mask_id):
    """All nodes reachable from the root along edges whose every new position passes A_pi."""
    K = len(S)

    def edge(p, k):
        if not S[p] < S[k]:
            return False
        live = [j for j in range(L) if drafts[p, block_start + j] == mask_id]
        return all(v_top1[p, j] == drafts[k, block_start + j] and commits_by_definition(v_conf[p], live, j, policy)
                   for j in S[k] - S[p])

    reachable = set()

    def walk(n):
        reachable.add(n)
        for k in range(K):
            if edge(n, k):
                walk(k)

    walk(0)
    best = max(len(S[k]) for k in reachable)
    k_star = min(k for k in reachable if len(S[k]) == best)
    return reachable, k_star


def random_graph(rng, K, max_rank):
    sets = {frozenset()}
    while len(sets) < K:
        size = int(rng.integers(1, max_rank + 1))
        sets.add(frozenset(int(r) for r in rng.choice(max_rank, size=size, replace=False)))
    ordered = sorted(sets, key=lambda s: (len(s), sorted(s)))
    return orc.Graph(tuple(ordered))


# ---------------------------------------------------------------- policy (Eq. 1, App. B.2)


def test_policy_matches_its_definition_position_by_position():
    rng = np.random.default_rng(0)
    for case in range(300):
        L = int(rng.integers(1, 20))
        conf = rng.random(L).astype(np.float32)
        if case % 3 == 0:
            conf = (np.floor(conf * 4) / 4).astype(np.float32)          # ties
        live = [j for j in range(L) if rng.random() < 0.7]
        policy = orc.Policy(tau=float(rng.choice([0.3, 0.9, INF, 0.0])), k_min=int(rng.integers(0, 4)),
                            k_max=int(rng.choice([0, 0, 1, 3])))
        T = orc.policy_select(live, conf, policy)
        assert set(T) == {i for i in live if commits_by_definition(conf, live, i, policy)}
        assert T == sorted(T, key=lambda i: (-conf[i], i))


def test_policy_monotone_in_tau_and_kmin_floor():
    rng = np.random.default_rng(1)
    for _ in range(100):
        L = 16
        conf = rng.random(L).astype(np.float32)
        live = list(range(L))
        sizes = [len(orc.policy_select(live, conf, orc.Policy(tau=t, k_min=1))) for t in (0.0, 0.3, 0.6, 0.9, INF)]
        assert sizes == sorted(sizes, reverse=True) and sizes[-1] == 1 and sizes[0] == L
        assert len(orc.policy_select(live, conf, orc.Policy(tau=INF, k_min=L))) == L
        for kmin in range(1, 5):
            assert len(orc.policy_select(live, conf, orc.Policy(tau=0.95, k_min=kmin))) >= kmin


def test_strictly_exceeds_threshold():
    conf = np.array([0.9, 0.9000001, 0.5], dtype=np.float32)
    T = orc.policy_select([0, 1, 2], conf, orc.Policy(tau=float(np.float32(0.9)), k_min=0))
    assert T == [1]


def test_select_unmask_changes_only_T_inside_the_block():
    for seed in range(50):
        tokens, top1, conf = inp.draw_block_state(seed, N=40, block_start=8, L=16, vocab=100)
        new, transfer = orc.select_unmask(tokens, 8, 16, top1, conf, orc.Policy(0.6, 1), 99)
        changed = np.nonzero(new != tokens)[0]
        assert set(changed) == {8 + j for j in range(16) if transfer[j]}
        for j in np.nonzero(transfer)[0]:
            assert tokens[8 + j] == 99 and new[8 + j] == top1[j]
        if (tokens[8:24] == 99).any():
            assert transfer.sum() >= 1


# ---------------------------------------------------------------- drafts (Eq. 2)


@pytest.mark.parametrize("K,width", [(1, 1), (2, 1), (4, 1), (8, 1), (4, 3)])
def test_draft_structure(K, width):
    graph = orc.chain_graph(K, width)
    for seed in range(40):
        tokens, top1, conf = inp.draw_block_state(seed, N=64, block_start=16, L=32, vocab=500,
                                                  tie_levels=5 if seed % 2 else 0)
        x1, _ = orc.select_unmask(tokens, 16, 32, top1, conf, orc.Policy(0.8, 1), 499)
        sigma, m, drafts = orc.build_drafts(x1, 16, 32, top1, conf, graph, 499)
        residual = [j for j in range(32) if x1[16 + j] == 499]
        assert m == len(residual) and sorted(sigma[:m]) == residual and (sigma[m:] == -1).all()
        cs = conf[sigma[:m]]
        assert (np.diff(cs) <= 0).all()
        for a, b in zip(sigma[:m - 1], sigma[1:m]):
            assert conf[a] > conf[b] or a < b                          # ties: lower position first
        assert (drafts[0] == x1).all()                                 # root = current state
        prev = set()
        for k in range(K):
            diff = {int(i) - 16 for i in np.nonzero(drafts[k] != x1)[0]}
            expect = set(int(s) for s in sigma[: min(m, k * width)])
            assert diff == expect and prev <= diff
            assert all(drafts[k, 16 + j] == top1[j] and x1[16 + j] == 499 for j in diff)
            prev = diff


def test_drafts_use_step_t_confidences_not_fresh_ones():
    # sigma must rank by the confidences handed in (step t), whatever the state is now
    tokens = np.array([5, 9, 9, 9, 9], dtype=np.int32)
    top1 = np.array([5, 1, 2, 3, 4], dtype=np.int32)
    conf = np.array([-1, 0.2, 0.8, 0.5, 0.8], dtype=np.float32)
    sigma, m, drafts = orc.build_drafts(tokens, 0, 5, top1, conf, orc.chain_graph(3), 9)
    assert m == 4 and list(sigma[:4]) == [2, 4, 3, 1]
    assert list(drafts[1]) == [5, 9, 2, 9, 9] and list(drafts[2]) == [5, 9, 2, 9, 4]


# ---------------------------------------------------------------- acceptance (Alg. 1 stage 3)


def _setup(seed, K=5, L=16, vocab=60, agree=0.8, graph=None, conf_kind="uniform", policy=None, stage1=None):
    policy = policy or orc.Policy(0.5, 1)
    tokens, top1, conf = inp.draw_block_state(seed, N=L + 8, block_start=4, L=L, vocab=vocab)
    x1, _ = orc.select_unmask(tokens, 4, L, top1, conf, stage1 or policy, vocab - 1)
    graph = graph or orc.chain_graph(K)
    sigma, m, drafts = orc.build_drafts(x1, 4, L, top1, conf, graph, vocab - 1)
    v_top1, v_conf = inp.draw_verifier_tables(seed + 1000, drafts, 4, L, vocab, top1, agree=agree, conf_kind=conf_kind)
    return x1, top1, conf, graph, sigma, m, drafts, v_top1, v_conf, policy


def test_full_agreement_is_accepted_at_full_depth_and_one_flip_cuts_it():
    policy = orc.Policy(tau=0.0, k_min=1)             # every positive confidence passes: pure token agreement
    hit = 0
    for seed in range(60):
        x1, top1, conf, graph, sigma, m, drafts, v_top1, v_conf, _ = _setup(seed, K=5, agree=1.0, policy=policy,
                                                                                  stage1=orc.Policy(INF, 1))
        if m < 4:
            continue
        hit += 1
        v_conf = np.where(v_conf >= 0, np.maximum(v_conf, 0.01), v_conf).astype(np.float32)
        acc, k_star = orc.hierarchical_accept(drafts, 4, 16, sigma, m, graph, policy, v_top1, v_conf, 59)
        assert acc.all() and k_star == 4
        # flip the verifier's token at the depth-3 position in every draft: depth <= 2
        j = int(sigma[2])
        bad = v_top1.copy()
        bad[:, j] = (bad[:, j] + 1) % 59
        acc, k_star = orc.hierarchical_accept(drafts, 4, 16, sigma, m, graph, policy, bad, v_conf, 59)
        assert k_star == 2 and list(acc) == [1, 1, 1, 0, 0]
        # flip it only in the root's and node 1's output: node 2 still vouches for node 3 and 4
        bad = v_top1.copy()
        bad[:2, j] = (bad[:2, j] + 1) % 59
        acc, k_star = orc.hierarchical_accept(drafts, 4, 16, sigma, m, graph, policy, bad, v_conf, 59)
        assert k_star == 4 and acc.all()
    assert hit > 20


@pytest.mark.parametrize("kind", ["chain", "wide-chain", "random-dag"])
def test_accepted_depth_is_the_deepest_consistent_one_by_brute_force(kind):
    rng = np.random.default_rng(42)
    depths = set()
    for seed in range(250):
        L = int(rng.integers(3, 9))
        K = int(rng.integers(2, 6))
        if kind == "chain":
            graph = orc.chain_graph(K)
        elif kind == "wide-chain":
            graph = orc.chain_graph(K, 2)
        else:
            graph = random_graph(rng, K, max_rank=4)
        policy = orc.Policy(tau=float(rng.choice([0.0, 0.4, 0.9, INF])), k_min=int(rng.integers(0, 3)),
                            k_max=int(rng.choice([0, 0, 2])))
        tokens, top1, conf = inp.draw_block_state(seed, N=L + 4, block_start=2, L=L, vocab=12, frac_masked=0.9,
                                                  tie_levels=4 if seed % 4 == 0 else 0)
        x1, _ = orc.select_unmask(tokens, 2, L, top1, conf, orc.Policy(INF, 1), 11)
        sigma, m, drafts = orc.build_drafts(x1, 2, L, top1, conf, graph, 11)
        v_top1, v_conf = inp.draw_verifier_tables(seed + 7, drafts, 2, L, 12, top1, agree=0.85)
        acc, k_star = orc.hierarchical_accept(drafts, 2, L, sigma, m, graph, policy, v_top1, v_conf, 11)
        S = orc.node_positions(graph, [int(s) for s in sigma[:m]])
        reach, k_bf = brute_force_accept(drafts, 2, L, S, policy, v_top1, v_conf, 11)
        assert {k for k in range(graph.K) if acc[k]} == reach
        assert k_star == k_bf
        depths.add(len(S[k_star]))
    assert len(depths) >= 3              # the cases really do span several depths


def test_root_always_accepted_and_duplicates_never_win():
    # fewer residual masks than the chain is deep: deeper nodes collapse onto the same set
    tokens = np.array([1, 9, 2, 9], dtype=np.int32)
    top1 = np.array([1, 4, 2, 6], dtype=np.int32)
    conf = np.array([-1, 0.3, -1, 0.6], dtype=np.float32)
    graph = orc.chain_graph(5)
    sigma, m, drafts = orc.build_drafts(tokens, 0, 4, top1, conf, graph, 9)
    assert m == 2 and (drafts[2] == drafts[3]).all() and (drafts[3] == drafts[4]).all()
    v_top1 = np.tile(top1, (5, 1))
    v_conf = np.where(drafts == 9, 0.99, -1).astype(np.float32)
    acc, k_star = orc.hierarchical_accept(drafts, 0, 4, sigma, m, graph, orc.Policy(0.9, 1), v_top1, v_conf, 9)
    # the collapsed copies are reachable exactly like node 2, but the lowest index wins the tie
    assert acc.all() and k_star == 2
    # hostile verifier: nothing agrees, only the root survives
    acc, k_star = orc.hierarchical_accept(drafts, 0, 4, sigma, m, graph, orc.Policy(0.9, 1), v_top1 + 1, v_conf, 9)
    assert list(acc) == [1, 0, 0, 0, 0] and k_star == 0


def test_advance_commits_policy_on_kstar_output():
    for seed in range(40):
        x1, top1, conf, graph, sigma, m, drafts, v_top1, v_conf, policy = _setup(seed)
        acc, k_star = orc.hierarchical_accept(drafts, 4, 16, sigma, m, graph, policy, v_top1, v_conf, 59)
        x2, n_post = orc.advance(drafts, k_star, 4, 16, v_top1, v_conf, policy, 59)
        live = [j for j in range(16) if drafts[k_star, 4 + j] == 59]
        expect = drafts[k_star].copy()
        for j in live:
            if commits_by_definition(v_conf[k_star], live, j, policy):
                expect[4 + j] = v_top1[k_star, j]
        assert (x2 == expect).all() and n_post == (expect != drafts[k_star]).sum()
        if live:
            assert n_post >= 1


# ---------------------------------------------------------------- whole-loop reductions


@pytest.mark.parametrize("K", [1, 2, 4, 8])
def test_greedy_policy_reproduces_plain_greedy_decoding(K):
    L, vocab = 12, 40
    for seed in range(12):
        fn = pseudo_model(vocab, seed, sticky=0.6)
        tokens = np.full(20, vocab - 1, dtype=np.int32)
        tokens[:8] = np.random.default_rng(seed).integers(0, vocab - 1, 8)
        ref, order = plain_greedy(fn, tokens, 8, L, vocab - 1)
        trace = []
        out, stats = orc.decode_block(fn, tokens, 8, L, orc.Policy(INF, 1), orc.chain_graph(K), vocab - 1, trace=trace)
        assert (out == ref).all()
        assert stats.tokens == L and stats.invocations <= L and stats.tpf >= 1.0
        if K == 1:
            assert [e[1][0] for e in trace if e[0] == "commit"][0] == order[0]


def test_greedy_reduction_on_the_real_tiny_model():
    w = inp.WORKLOADS[1]
    model = inp.draw_model(w.shape, w.seq_len)
    fn = orc.model_confidence_fn(model)
    tokens = inp.initial_state(w)[0]
    ref, _ = plain_greedy(fn, tokens, w.prompt_len, 8, w.shape.mask_id)
    for K in (1, 3):
        out, stats = orc.decode_block(fn, tokens, w.prompt_len, 8, orc.Policy(INF, 1), orc.chain_graph(K),
                                      w.shape.mask_id)
        assert (out == ref).all() and stats.tokens == 8 and stats.tpf >= 1.0


@pytest.mark.parametrize("tau", [0.5, 0.9])
def test_root_only_graph_is_plain_parallel_decoding(tau):
    L, vocab = 16, 50
    for seed in range(15):
        fn = Counting(pseudo_model(vocab, seed))
        tokens = np.full(24, vocab - 1, dtype=np.int32)
        tokens[:8] = 3
        ref, calls = plain_parallel(fn, tokens, 8, L, vocab - 1, tau)
        out, stats = orc.decode_block(pseudo_model(vocab, seed), tokens, 8, L, orc.Policy(tau, 1),
                                      orc.chain_graph(1), vocab - 1)
        # with K = 1 each iteration is: stage-1 commit, then the root "verification" whose own
        # output is committed by the same policy -- i.e. two plain parallel steps
        assert (out == ref).all()
        assert stats.invocations == calls


def test_progress_termination_and_tpf():
    L, vocab = 32, 200
    for seed in range(20):
        for K, tau, kind in ((4, 0.9, "uniform"), (8, 0.9, "low"), (2, 0.3, "uniform")):
            fn = Counting(pseudo_model(vocab, seed, conf_kind=kind, sticky=0.7))
            tokens = np.full(48, vocab - 1, dtype=np.int32)
            tokens[:16] = 1
            trace = []
            out, stats = orc.decode_block(fn, tokens, 16, L, orc.Policy(tau, 1), orc.chain_graph(K), vocab - 1,
                                          trace=trace)
            assert not (out[16:48] == vocab - 1).any() and (out[:16] == 1).all()
            assert stats.tokens == L and stats.invocations <= L and stats.tpf >= 1.0
            assert sum(stats.depth_hist) == sum(1 for e in trace if e[0] == "verify")
            n_verify = sum(stats.depth_hist)
            assert fn.calls == (stats.invocations - n_verify) + K * n_verify   # a batched verify = 1 invocation


def test_speculation_pays_when_predictions_are_stable():
    # fully state-independent predictions: every draft is right, chains are accepted whole
    vocab, L = 30, 16
    fn = pseudo_model(vocab, 3, conf_kind="low", sticky=1.0)
    tokens = np.full(L, vocab - 1, dtype=np.int32)
    _, s1 = orc.decode_block(fn, tokens, 0, L, orc.Policy(0.9, 1), orc.chain_graph(1), vocab - 1)
    _, s4 = orc.decode_block(fn, tokens, 0, L, orc.Policy(0.9, 1), orc.chain_graph(4), vocab - 1)
    assert s1.tpf == 1.0
    assert s4.tpf == pytest.approx(16 / 7)      # 5 tokens per 2 invocations, last token alone
    assert s4.depth_hist[3] == 3


def test_hand_worked_chain_trace_fixture():
    """tests/golden/chain_trace.txt: Alg. 1 worked by hand for a model whose predictions never change (every draft
    is right).  The oracle's trace must reproduce it iteration by iteration."""
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "chain_trace.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    vocab, L = 30, 16
    fn = pseudo_model(vocab, 3, conf_kind="low", sticky=1.0)
    tokens = np.full(L, vocab - 1, dtype=np.int32)
    trace = []
    _, stats = orc.decode_block(fn, tokens, 0, L, orc.Policy(0.9, 1), orc.chain_graph(4), vocab - 1, trace=trace)
    got, masks, i = [], L, 0
    while i < len(trace):
        assert trace[i][0] == "commit"
        n1 = len(trace[i][1])
        if i + 1 < len(trace) and trace[i + 1][0] == "verify":
            _, _, depth, n_post, _ = trace[i + 1]
            got.append([str(len(got) + 1), str(masks), str(n1), str(depth), str(n_post), "2"])
            masks -= n1 + depth + n_post
            i += 2
        else:
            got.append([str(len(got) + 1), str(masks), str(n1), "-", "-", "1"])
            masks -= n1
            i += 1
    assert got == rows
    assert masks == 0 and stats.tokens == 16 and stats.invocations == 7


def test_blocks_decode_left_to_right_and_later_blocks_stay_masked():
    vocab, L = 30, 8
    seen = []

    def fn(tokens, block_start, Lb):
        seen.append((block_start, int((np.asarray(tokens)[block_start + Lb:] == vocab - 1).all())))
        return pseudo_model(vocab, 5)(tokens, block_start, Lb)

    tokens = np.full(4 + 3 * L, vocab - 1, dtype=np.int32)
    tokens[:4] = 2
    out, stats = orc.decode(fn, tokens, 4, L, orc.Policy(0.9, 1), orc.chain_graph(2), vocab - 1)
    assert not (out == vocab - 1).any() and stats.tokens == 3 * L
    starts = [s for s, _ in seen]
    assert starts == sorted(starts) and set(starts) == {4, 12, 20} and all(flag for _, flag in seen)


# ---------------------------------------------------------------- EOS early stopping (App. B.1)


def scripted_model(top1, conf, mask_id):
    """Predictions that never depend on the state (every draft is right)."""
    top1, conf = np.asarray(top1, dtype=np.int32), np.asarray(conf, dtype=np.float32)

    def fn(tokens, block_start, L):
        blk = np.asarray(tokens[block_start: block_start + L])
        masked = blk == mask_id
        return np.where(masked, top1, blk).astype(np.int32), np.where(masked, conf, np.float32(-1)).astype(np.float32)

    return fn


def test_eos_stop_hand_worked():
    """L = 8, chain K = 3 (depths 0, 1, 2), tau = 0.9, k_min = 1, all confidences below tau.
    Iteration 1 by hand: stage 1 commits position 3 (0.8).  sigma = 1 (0.5), 2 (0.3), 4 (0.2), ...; drafts fill
    {}, {1}, {1, 2}.  The predictions never change, so on the root's output the policy commits position 1 and on
    the depth-1 draft's output position 2: both edges pass, k* is the depth-2 draft.  The post-verification
    commit on its output takes position 4 (0.2).  State after the iteration: positions 1, 2, 3, 4 resolved."""
    mask, eos, L = 99, 9, 8
    conf = [0.1, 0.5, 0.3, 0.8, 0.2, 0.05, 0.04, 0.03]
    P = 4                                        # a resolved prompt in front: positions below are block-local
    tokens = np.full(P + L, mask, dtype=np.int32)
    tokens[:P] = 7
    policy, graph = orc.Policy(0.9, 1), orc.chain_graph(3)
    # EOS predicted at position 2: it is produced by the accepted draft of iteration 1 -> stop after 2 invocations;
    # positions at or before it that were resolved: 1 and 2 (0 is still masked; 3 and 4 lie beyond and are discarded)
    fn = Counting(scripted_model([5, 5, eos, 5, 5, 5, 5, 5], conf, mask))
    out, st = orc.decode_block(fn, tokens, P, L, policy, graph, mask, eos_id=eos)
    assert out.tolist() == [7] * P + [mask, 5, eos, 5, 5, mask, mask, mask]
    assert (st.stopped, st.eos_pos, st.invocations, st.tokens_counted) == (True, P + 2, 2, 2)
    assert (st.tokens_policy, st.tokens_draft, st.tokens_postverify) == (1, 2, 1) and st.tpf_counted == 1.0
    assert fn.calls == 1 + 3
    # EOS predicted at position 3: the stage-1 commit produces it -> stop before any verification call
    fn = Counting(scripted_model([5, 5, 5, eos, 5, 5, 5, 5], conf, mask))
    out, st = orc.decode_block(fn, tokens, P, L, policy, graph, mask, eos_id=eos)
    assert out.tolist() == [7] * P + [mask, mask, mask, eos, mask, mask, mask, mask]
    assert (st.stopped, st.eos_pos, st.invocations, st.tokens_counted, fn.calls) == (True, P + 3, 1, 1, 1)
    # EOS predicted at position 4: produced by the post-verification commit; resolved at or before it: 1, 2, 3, 4
    fn = scripted_model([5, 5, 5, 5, eos, 5, 5, 5], conf, mask)
    out, st = orc.decode_block(fn, tokens, P, L, policy, graph, mask, eos_id=eos)
    assert (st.stopped, st.eos_pos, st.invocations, st.tokens_counted) == (True, P + 4, 2, 4)
    # the same model without early stopping resolves the block and counts every token
    out, st = orc.decode_block(fn, tokens, P, L, policy, graph, mask)
    assert not (out == mask).any() and (st.stopped, st.eos_pos, st.tokens_counted) == (False, -1, L) and st.tokens == L
    with pytest.raises(ValueError):
        orc.decode_block(fn, tokens, P, L, policy, graph, mask, eos_id=mask)


def test_eos_that_never_appears_changes_nothing():
    vocab, L = 200, 32
    for seed in range(6):
        fn = pseudo_model(vocab, seed, sticky=0.7)
        tokens = np.full(48, vocab - 1, dtype=np.int32)
        tokens[:16] = 1
        a, sa = orc.decode_block(fn, tokens, 16, L, orc.Policy(0.9, 1), orc.chain_graph(4), vocab - 1)
        b, sb = orc.decode_block(fn, tokens, 16, L, orc.Policy(0.9, 1), orc.chain_graph(4), vocab - 1, eos_id=vocab + 7)
        assert (a == b).all() and not sb.stopped and sb.tokens_counted == sb.tokens == L
        assert (sa.invocations, sa.tokens_policy, sa.tokens_draft, sa.tokens_postverify) == \
               (sb.invocations, sb.tokens_policy, sb.tokens_draft, sb.tokens_postverify)


def test_eos_stop_is_the_first_state_with_an_eos_on_the_free_trajectory():
    """The stopped run must walk the free run's trajectory (same commits, same values) and end at the first state
    update after which the block holds the EOS token: no earlier state that the model was called on -- the input
    of a stage-1 call, or the root draft of a verification batch, which is the state after the stage-1 commit --
    may contain it, and the final state must."""
    vocab, L, K, start = 200, 32, 4, 16
    mask = vocab - 1
    stopped_midway = 0
    for seed in range(12):
        base = pseudo_model(vocab, seed, sticky=0.7)
        tokens = np.full(48, mask, dtype=np.int32)
        tokens[:16] = 1
        free, sf = orc.decode_block(base, tokens, start, L, orc.Policy(0.9, 1), orc.chain_graph(K), mask)
        eos = int(free[start + 5 + seed])          # a token the free run does produce
        calls = []

        def fn(t, bs, Lb):
            calls.append(np.array(t, copy=True))
            return base(t, bs, Lb)

        out, st = orc.decode_block(fn, tokens, start, L, orc.Policy(0.9, 1), orc.chain_graph(K), mask, eos_id=eos)
        blk = out[start:start + L]
        assert st.stopped and eos in blk.tolist() and st.eos_pos == start + blk.tolist().index(eos)
        resolved = blk != mask
        assert (blk[resolved] == free[start:start + L][resolved]).all()
        assert st.invocations <= sf.invocations
        for i, state in enumerate(calls):           # calls come in groups: stage 1, then the K drafts (root first)
            if i % (K + 1) in (0, 1):
                assert eos not in state[start:start + L].tolist()
        assert st.tokens_counted == int(resolved[: st.eos_pos - start + 1].sum())
        assert 1 <= st.tokens_counted <= st.tokens
        stopped_midway += int((blk == mask).any())
    assert stopped_midway >= 6                      # the stop does cut decoding short


def test_eos_ends_the_generation_after_its_block():
    vocab, L, mask = 30, 8, 29
    base = pseudo_model(vocab, 5)
    tokens = np.full(4 + 3 * L, mask, dtype=np.int32)
    tokens[:4] = 2
    free, _ = orc.decode(base, tokens, 4, L, orc.Policy(0.9, 1), orc.chain_graph(2), mask)
    eos = int(free[4 + L + 3])                       # first produced in the second block (checked below)
    assert eos not in free[4:4 + L].tolist()
    out, st = orc.decode(base, tokens, 4, L, orc.Policy(0.9, 1), orc.chain_graph(2), mask, eos_id=eos)
    assert (out[4:4 + L] == free[4:4 + L]).all() and st.stopped and 4 + L <= st.eos_pos < 4 + 2 * L
    assert (out[4 + 2 * L:] == mask).all()
    assert st.tokens_counted == L + int((out[4 + L: st.eos_pos + 1] != mask).sum())


# ---------------------------------------------------------------- the single-forward variant


@pytest.mark.parametrize("tau", [0.5, 0.9])
def test_single_forward_with_the_root_only_graph_is_plain_parallel_decoding(tau):
    """K = 1: every call, the first included, is a forward on the current state followed by the policy's commit."""
    L, vocab = 16, 50
    for seed in range(15):
        tokens = np.full(24, vocab - 1, dtype=np.int32)
        tokens[:8] = 3
        ref, calls = plain_parallel(pseudo_model(vocab, seed), tokens, 8, L, vocab - 1, tau)
        fn = Counting(pseudo_model(vocab, seed))
        out, stats = orc.decode_block(fn, tokens, 8, L, orc.Policy(tau, 1), orc.chain_graph(1), vocab - 1, single_forward=True)
        assert (out == ref).all()
        assert stats.invocations == calls == fn.calls


@pytest.mark.parametrize("K", [1, 2, 4, 8])
def test_single_forward_with_the_greedy_policy_reproduces_plain_greedy_decoding(K):
    """Every commit of the variant is taken from an exact forward of an exact state, and with greedy pi the acceptance
    criterion lets through exactly what greedy decoding would reveal next: same tokens, fewer calls."""
    L, vocab = 12, 40
    fewer = 0
    for seed in range(12):
        fn = pseudo_model(vocab, seed, sticky=0.6)
        tokens = np.full(20, vocab - 1, dtype=np.int32)
        tokens[:8] = np.random.default_rng(seed).integers(0, vocab - 1, 8)
        ref, _ = plain_greedy(fn, tokens, 8, L, vocab - 1)
        out, stats = orc.decode_block(fn, tokens, 8, L, orc.Policy(INF, 1), orc.chain_graph(K), vocab - 1, single_forward=True)
        _, literal = orc.decode_block(fn, tokens, 8, L, orc.Policy(INF, 1), orc.chain_graph(K), vocab - 1)
        assert (out == ref).all()
        assert stats.tokens == L and stats.invocations <= L and stats.tpf >= 1.0
        fewer += int(stats.invocations < literal.invocations)
    assert K == 1 or fewer > 0


def test_single_forward_progress_calls_and_first_iteration():
    L, vocab = 32, 200
    for seed in range(20):
        for K, tau, kind in ((4, 0.9, "uniform"), (8, 0.9, "low"), (2, 0.3, "uniform")):
            tokens = np.full(48, vocab - 1, dtype=np.int32)
            tokens[:16] = 1
            fn = Counting(pseudo_model(vocab, seed, conf_kind=kind, sticky=0.7))
            trace = []
            out, stats = orc.decode_block(fn, tokens, 16, L, orc.Policy(tau, 1), orc.chain_graph(K), vocab - 1, trace=trace,
                                          single_forward=True)
            assert not (out[16:48] == vocab - 1).any() and (out[:16] == 1).all()
            n_verify = sum(stats.depth_hist)
            assert stats.tokens == L and stats.tpf >= 1.0
            assert stats.invocations == 1 + n_verify                 # one stage-1 call per block, then verifications only
            assert fn.calls == 1 + K * n_verify
            assert [e[0] for e in trace] == ["commit"] + ["verify"] * n_verify
            # up to and including the first verification the variant IS the literal loop
            lit = []
            orc.decode_block(pseudo_model(vocab, seed, conf_kind=kind, sticky=0.7), tokens, 16, L, orc.Policy(tau, 1),
                             orc.chain_graph(K), vocab - 1, trace=lit)
            assert trace[0] == lit[0]
            if n_verify:
                assert trace[1][1:4] == lit[1][1:4] and (trace[1][4] == lit[1][4]).all()


def test_single_forward_refreshes_its_tables_with_every_new_block_and_stops_on_eos():
    vocab, L = 60, 8
    fn = Counting(pseudo_model(vocab, 11, sticky=0.5))
    tokens = np.full(4 + 3 * L, vocab - 1, dtype=np.int32)
    tokens[:4] = 2
    out, stats = orc.decode(fn, tokens, 4, L, orc.Policy(0.9, 1), orc.chain_graph(3), vocab - 1, single_forward=True)
    assert not (out == vocab - 1).any()
    n_verify = sum(stats.depth_hist)
    assert stats.invocations == 3 + n_verify and fn.calls == 3 + 3 * n_verify        # one stage-1 call per block
    eos = int(out[4 + L + 2])
    cut, st = orc.decode(pseudo_model(vocab, 11, sticky=0.5), tokens, 4, L, orc.Policy(0.9, 1), orc.chain_graph(3), vocab - 1,
                         eos_id=eos, single_forward=True)
    assert st.stopped and cut[st.eos_pos] == eos and st.eos_pos <= 4 + L + 2
    assert (cut[4 + ((st.eos_pos - 4) // L + 1) * L:] == vocab - 1).all()


def test_single_forward_hand_worked_trace_fixture():
    """tests/golden/single_forward_trace.txt, worked by hand from the variant's definition."""
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "single_forward_trace.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(line.split())
    vocab, L = 30, 16
    fn = pseudo_model(vocab, 3, conf_kind="low", sticky=1.0)
    tokens = np.full(L, vocab - 1, dtype=np.int32)
    trace = []
    out, stats = orc.decode_block(fn, tokens, 0, L, orc.Policy(0.9, 1), orc.chain_graph(4), vocab - 1, trace=trace, single_forward=True)
    got, masks = [], L
    for n, e in enumerate(trace, 1):
        if e[0] == "commit":
            got.append([str(n), str(masks), "stage1", str(len(e[1])), "-", "-"])
            masks -= len(e[1])
        else:
            _, _, depth, n_post, _ = e
            got.append([str(n), str(masks), "verify", "-", str(depth), str(n_post)])
            masks -= depth + n_post
    assert got == rows
    assert masks == 0 and stats.tokens == 16 and stats.invocations == 5
    literal, _ = orc.decode_block(fn, tokens, 0, L, orc.Policy(0.9, 1), orc.chain_graph(4), vocab - 1)
    assert (out == literal).all()            # predictions never change here: same tokens, 5 calls instead of 7
