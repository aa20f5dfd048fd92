"""End-to-end parity of the PSD loop with the oracle, through the C ABI.

fp32 (config 1): free-running decode, tokens and counters must match exactly.
bf16: lock-step.  Both sides start every iteration from the same state; the GPU's (top1, conf)
tables feed the oracle's decision functions, which must reproduce the GPU's decisions bit for
bit; the model outputs are compared with the oracle's own forward away from near-ties (oracle
top-1 margin, distance to tau and adjacent confidence gaps below the guard are logged; both
sides then continue from the one state reached with the GPU's tables, so a near-tie never
voids the rest of the run)."""
import numpy as np
import pytest
import torch

import psd_inputs as inp
from oracle import psd_oracle as orc
from tests import parity_guard as G

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def test_config1_free_running_decode_matches_oracle_exactly():
    import paper_2605_15609_amd as psd
    w = inp.WORKLOADS[1]
    host = inp.draw_model(w.shape, w.seq_len)
    model = psd.Model.from_host(host, DEV)
    for K, tau in ((2, 0.9), (4, 0.02), (1, 0.9), (3, float("inf"))):
        tokens0 = inp.initial_state(w)
        d_tokens = _dev(tokens0)
        stats = psd.decode(model, d_tokens, w.prompt_len, w.block_len, psd.Policy(tau, 1, 0), psd.chain_graph(K))
        ref, ostats = orc.decode(orc.model_confidence_fn(host), tokens0[0], w.prompt_len, w.block_len,
                                 orc.Policy(tau, 1, 0), orc.chain_graph(K), w.shape.mask_id)
        assert (d_tokens.cpu().numpy()[0] == ref).all(), (K, tau)
        s = stats[0]
        assert (s.invocations, s.tokens_policy, s.tokens_draft, s.tokens_postverify) == \
               (ostats.invocations, ostats.tokens_policy, ostats.tokens_draft, ostats.tokens_postverify)
        assert s.depth_hist[:32] == ostats.depth_hist and s.tpf >= 1.0


def test_decode_block_equals_the_step_calls_composed():
    """psd_decode_block must be exactly the four step calls in Alg. 1's order (same kernels)."""
    import paper_2605_15609_amd as psd
    shape = inp.cut_down(inp.WORKLOADS[2].shape, n_layers=2, vocab=4000, seed=31)
    N, P, L, K = 160, 64, 32, 4
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    policy, graph = psd.Policy(0.9, 1, 0), psd.chain_graph(K)
    tokens = np.full((1, N), shape.mask_id, dtype=np.int32)
    tokens[0, :P] = inp.draw_prompt(shape.vocab, P, 5)
    a = _dev(tokens)
    stats = psd.psd_decode_block(model, a, P, L, policy, graph)
    b = _dev(tokens)
    inv = 0
    while bool((b[0, P:P + L] == shape.mask_id).any()):
        top1, conf = psd.psd_forward_confidence(model, b, P, L)
        inv += 1
        psd.psd_select_unmask(model, b, P, L, top1, conf, policy)
        sigma, m, drafts = psd.psd_build_drafts(model, b, P, L, top1, conf, graph)
        if int(m[0]) == 0:
            break
        psd.psd_verify_accept(model, b, drafts, P, L, sigma, m, graph, policy)
        inv += 1
    assert (a == b).all() and stats[0].invocations == inv and stats[0].tokens == L


def test_batched_decode_equals_sequences_decoded_alone():
    import paper_2605_15609_amd as psd
    shape = inp.cut_down(inp.WORKLOADS[2].shape, n_layers=2, vocab=4000, seed=32, logit_scale=14.0)
    N, P, L, K, B = 136, 40, 32, 3, 5
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    policy, graph = psd.Policy(0.9, 1, 0), psd.chain_graph(K)
    tokens = np.full((B, N), shape.mask_id, dtype=np.int32)
    for b in range(B):
        tokens[b, :P] = inp.draw_prompt(shape.vocab, P, 50 + b)
    tokens[3, P: P + L] = 7                     # one sequence arrives with its block already resolved
    together = _dev(tokens)
    stats = psd.decode(model, together, P, L, policy, graph)
    for b in range(B):
        alone = _dev(tokens[b: b + 1])
        s = psd.decode(model, alone, P, L, policy, graph)
        assert (alone[0] == together[b]).all(), b
        assert (s[0].invocations, s[0].tokens) == (stats[b].invocations, stats[b].tokens)
    assert not bool((together == shape.mask_id).any())
    assert stats[3].invocations < stats[0].invocations
    assert all(s.tpf >= 1.0 for s in stats)


def _counters(s):
    return (s.invocations, s.tokens_policy, s.tokens_draft, s.tokens_postverify, s.tokens_counted, bool(s.stopped), s.eos_pos)


def test_config1_eos_early_stop_matches_oracle_exactly():
    """App. B.1: stop as soon as an EOS token is produced, count the tokens up to and including its position.
    The EOS ids are tokens the oracle's free run produces at chosen positions, so the stop falls early, in the
    middle and late in the block; three sequences share a batch, so the others go on while one has stopped."""
    import paper_2605_15609_amd as psd
    w = inp.WORKLOADS[1]
    shape, P, L = w.shape, w.prompt_len, w.block_len
    host = inp.draw_model(shape, w.seq_len)
    model = psd.Model.from_host(host, DEV)
    fn = orc.model_confidence_fn(host)
    B = 3
    tokens0 = np.full((B, w.seq_len), shape.mask_id, dtype=np.int32)
    for b in range(B):
        tokens0[b, :P] = inp.draw_prompt(shape.vocab, P, 300 + b)
    cut_short = 0
    for K, tau in ((2, 0.9), (4, 0.02)):
        free = [orc.decode(fn, tokens0[b], P, L, orc.Policy(tau, 1, 0), orc.chain_graph(K), shape.mask_id)[0] for b in range(B)]
        for pick in (1, 13, 30):
            eos = int(free[0][P + pick])
            d_tokens = _dev(tokens0)
            stats = psd.decode(model, d_tokens, P, L, psd.Policy(tau, 1, 0, eos_id=eos), psd.chain_graph(K))
            got = d_tokens.cpu().numpy()
            for b in range(B):
                ref, ost = orc.decode(fn, tokens0[b], P, L, orc.Policy(tau, 1, 0), orc.chain_graph(K), shape.mask_id, eos_id=eos)
                assert (got[b] == ref).all(), (K, tau, pick, b)
                assert _counters(stats[b]) == _counters(ost), (K, tau, pick, b)
                cut_short += int(ost.stopped and (ref == shape.mask_id).any())
            assert stats[0].stopped
        # an EOS id that is never produced: nothing changes, every token counts
        unused = next(t for t in range(shape.vocab) if t != shape.mask_id and all(t not in f.tolist() for f in free))
        d_tokens = _dev(tokens0)
        stats = psd.decode(model, d_tokens, P, L, psd.Policy(tau, 1, 0, eos_id=unused), psd.chain_graph(K))
        for b in range(B):
            assert (d_tokens.cpu().numpy()[b] == free[b]).all() and not stats[b].stopped
            assert stats[b].tokens_counted == stats[b].tokens == L
    assert cut_short >= 3


def test_eos_stop_in_a_batch_over_several_blocks_equals_sequences_alone():
    import paper_2605_15609_amd as psd
    shape = inp.cut_down(inp.WORKLOADS[2].shape, n_layers=2, vocab=4000, seed=32, logit_scale=14.0)
    N, P, L, K, B = 136, 40, 32, 3, 5
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    graph = psd.chain_graph(K)
    tokens = np.full((B, N), shape.mask_id, dtype=np.int32)
    for b in range(B):
        tokens[b, :P] = inp.draw_prompt(shape.vocab, P, 50 + b)
    free = _dev(tokens)
    psd.decode(model, free, P, L, psd.Policy(0.9, 1, 0), graph)
    eos = int(free[1, P + L + 9])               # produced by sequence 1 in its second block (if not before)
    policy = psd.Policy(0.9, 1, 0, eos_id=eos)
    together = _dev(tokens)
    stats = psd.decode(model, together, P, L, policy, graph)
    for b in range(B):
        alone = _dev(tokens[b: b + 1])
        s = psd.decode(model, alone, P, L, policy, graph)
        assert (alone[0] == together[b]).all(), b
        assert _counters(s[0]) == _counters(stats[b]), b
        row = together[b].cpu().numpy()
        if stats[b].stopped:
            assert row[stats[b].eos_pos] == eos and eos not in row[P:stats[b].eos_pos].tolist()
            nxt = P + ((stats[b].eos_pos - P) // L + 1) * L
            assert (row[nxt:] == shape.mask_id).all()           # no block after the one with the EOS was started
            assert stats[b].tokens_counted <= stats[b].tokens
        else:
            assert eos not in row[P:].tolist() and not (row == shape.mask_id).any()
            assert stats[b].tokens_counted == stats[b].tokens == N - P
    assert stats[1].stopped and stats[1].eos_pos < P + 2 * L
    assert any(not s.stopped for s in stats)


def test_graph_calibration_scores_every_candidate_like_the_oracle():
    """Offline choice of the draft graph (Sec. 3.2 stage 2): every candidate's tokens, invocations and TPF on the
    calibration batch must be the oracle's for that graph (fp32 model, exact); the winner is the candidate with the
    highest measured tokens per second; the batch itself is left untouched."""
    import paper_2605_15609_amd as psd
    w = inp.WORKLOADS[1]
    shape, P, L = w.shape, w.prompt_len, w.block_len
    host = inp.draw_model(shape, w.seq_len)
    model = psd.Model.from_host(host, DEV)
    fn = orc.model_confidence_fn(host)
    B = 2
    tokens0 = np.full((B, w.seq_len), shape.mask_id, dtype=np.int32)
    for b in range(B):
        tokens0[b, :P] = inp.draw_prompt(shape.vocab, P, 400 + b)
    cands = [psd.chain_graph(1), psd.chain_graph(2), psd.chain_graph(4), psd.chain_graph(3, 2), psd.lattice_graph(2),
             psd.lattice_graph(3), psd.Graph((0, 1, 2, 3, 6))]
    d = _dev(tokens0)
    best, scores = psd.psd_calibrate_graph(model, d, P, L, psd.Policy(0.05, 1, 0), cands)
    assert (d.cpu().numpy() == tokens0).all()
    for g, sc in zip(cands, scores):
        og = orc.Graph(tuple(frozenset(r for r in range(64) if (rs >> r) & 1) for rs in g.rank_sets))
        tok = inv = 0
        for b in range(B):
            _, st = orc.decode(fn, tokens0[b], P, L, orc.Policy(0.05, 1, 0), og, shape.mask_id)
            tok, inv = tok + st.tokens, inv + st.invocations
        assert (sc["tokens"], sc["invocations"]) == (tok, inv) and tok == B * (w.seq_len - P), g.rank_sets
        assert sc["tpf"] == pytest.approx(tok / inv) and sc["seconds"] > 0
        assert sc["tokens_per_s"] == pytest.approx(tok / sc["seconds"])
    assert best == max(range(len(cands)), key=lambda c: (scores[c]["tokens_per_s"], -c))
    with pytest.raises(psd.PsdError):
        psd.psd_calibrate_graph(model, d, P + 1, L, psd.Policy(), cands)        # generated part not whole blocks


def _check_tables(host, tokens_rows, bs, L, g_top1, g_conf, log, guard, eps):
    """GPU model output vs oracle model output on the same states (one oracle forward per row of tokens_rows);
    returns per row (oracle top1, oracle conf, near-tie flags, oracle top-1 margins)."""
    shape = host.shape
    mask_id = shape.mask_id
    out = []
    for r, t in enumerate(tokens_rows):
        o_top1, o_conf, z = orc.forward_confidence(host, t, bs, L, return_logits=True)
        masked = t[bs: bs + L] == mask_id
        zz = z.copy()
        zz[:, mask_id] = -np.inf
        part = np.partition(zz, -2, axis=-1)
        margin = part[:, -1] - part[:, -2]
        tie = masked & (margin < guard)
        log["near_tie_top1"] += int(tie.sum())
        # A logit error of eps on either side lets the argmax land on any token whose oracle logit
        # is within 2*eps of the top one.  Positions with margin < 1e-3 are the logged near-ties;
        # a mismatch beyond that must still stay inside the band the logit tolerance implies.
        differ = masked & (g_top1[r] != o_top1)
        for j in np.nonzero(differ)[0]:
            gap = zz[j, o_top1[j]] - zz[j, g_top1[r][j]]
            assert gap <= 2 * eps, f"top-1 mismatch with oracle logit gap {gap:.3e} > 2 * {eps}"
            if margin[j] >= guard:
                log["top1_within_logit_tol"] = log.get("top1_within_logit_tol", 0) + 1
        ok = masked & ~differ
        assert (g_top1[r][~masked] == o_top1[~masked]).all() and (g_conf[r][~masked] == -1).all()
        if ok.any():
            rel = np.abs(g_conf[r][ok] / o_conf[ok] - 1).max()
            log["max_conf_rel"] = max(log["max_conf_rel"], float(rel))
            assert rel < np.expm1(2 * eps), f"confidence off by {rel}"
        out.append((o_top1, o_conf, tie, margin))
    return out


def _lockstep(workload, shape, n_blocks, guard=1e-3, max_iters=10 ** 9):
    import paper_2605_15609_amd as psd
    from tests.gpu_common import gpu_graph
    N, P, L, K = workload.seq_len, workload.prompt_len, workload.block_len, workload.n_drafts
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    opol, ograph = orc.Policy(workload.tau, workload.k_min, workload.k_max), orc.chain_graph(K)
    gpol, ggraph = psd.Policy(workload.tau, workload.k_min, workload.k_max), gpu_graph(ograph)
    mask_id = shape.mask_id
    x = inp.initial_state(workload)[0]
    log = {"iters": 0, "near_tie_top1": 0, "commit_sets_differ": 0, "rank_pairs_inverted": 0, "verdicts_differ": 0,
           "resync": 0, "unexplained": 0, "max_conf_rel": 0.0}
    eps_logit = 2e-2 * max(1.0, shape.logit_scale)
    r_conf = float(np.expm1(2 * eps_logit))       # relative confidence error that a logit error of eps_logit allows
    n_ranks = max(max(rs) + 1 if rs else 0 for rs in ograph.rank_sets)     # ranks of sigma that feed the drafts

    def check_tables(tokens_rows, g_top1, g_conf):
        return _check_tables(host, tokens_rows, bs, L, g_top1, g_conf, log, guard, eps_logit)

    for blk in range(n_blocks):
        bs = P + blk * L
        while (x[bs: bs + L] == mask_id).any() and log["iters"] < max_iters:
            log["iters"] += 1
            d_x = _dev(x[None])
            g_top1, g_conf = psd.psd_forward_confidence(model, d_x, bs, L)
            g_top1_h, g_conf_h = g_top1.cpu().numpy(), g_conf.cpu().numpy()
            (o_top1, o_conf, _, _), = check_tables([x], g_top1_h, g_conf_h)
            # decisions: same tables in -> identical decisions out (no exclusions)
            tm, ns = psd.psd_select_unmask(model, d_x, bs, L, g_top1, g_conf, gpol)
            sigma, m, drafts = psd.psd_build_drafts(model, d_x, bs, L, g_top1, g_conf, ggraph)
            x1, o_tm = orc.select_unmask(x, bs, L, g_top1_h[0], g_conf_h[0], opol, mask_id)
            assert (d_x.cpu().numpy()[0] == x1).all() and (tm.cpu().numpy()[0] == o_tm).all()
            o_sigma, o_m, o_drafts = orc.build_drafts(x1, bs, L, g_top1_h[0], g_conf_h[0], ograph, mask_id)
            assert int(m[0]) == o_m and (sigma.cpu().numpy()[0] == o_sigma).all()
            assert (drafts.cpu().numpy()[0] == o_drafts).all()
            # would the oracle, on its own tables, have decided the same?  Only the pairs whose order actually
            # differs (and threshold crossings) may be blamed, and only when they are near-ties.
            x1_o, _ = orc.select_unmask(x, bs, L, o_top1, o_conf, opol, mask_id)
            s_o, m_o, d_o = orc.build_drafts(x1_o, bs, L, o_top1, o_conf, ograph, mask_id)
            T_g = [j for j in range(L) if x1[bs + j] != x[bs + j]]
            T_o = [j for j in range(L) if x1_o[bs + j] != x[bs + j]]
            bad = G.unexplained_commit_differences(o_conf, T_o, T_g, opol.tau, r_conf)
            log["commit_sets_differ"] += int(set(T_o) != set(T_g))
            # a committed position whose top-1 differs is the top-1 rule's business (checked in check_tables)
            if set(T_o) == set(T_g):
                inv = G.inverted_pairs(list(s_o[:m_o]), list(o_sigma[:o_m]), n_ranks)
                log["rank_pairs_inverted"] += len(inv)
                bad += [("rank", p) for p in G.unexplained_rank_differences(o_conf, s_o[:m_o], o_sigma[:o_m], n_ranks, r_conf)]
            log["unexplained"] += len(bad)
            assert not bad, f"decision differs from the oracle's without a near-tie on the pairs involved: {bad}"
            if not ((x1_o == x1).all() and (d_o == o_drafts).all()):
                log["resync"] += 1      # both sides continue from the common state reached with the GPU's tables
            if o_m == 0:
                x = x1
                continue
            k_star, accepted, v_top1, v_conf = psd.psd_verify_accept(model, d_x, drafts, bs, L, sigma, m, ggraph, gpol)
            v_top1_h, v_conf_h = v_top1.cpu().numpy()[0], v_conf.cpu().numpy()[0]
            o_tabs = check_tables(list(o_drafts), v_top1_h, v_conf_h)
            o_acc, o_k = orc.hierarchical_accept(o_drafts, bs, L, o_sigma, o_m, ograph, opol, v_top1_h, v_conf_h, mask_id)
            x2, _ = orc.advance(o_drafts, o_k, bs, L, v_top1_h, v_conf_h, opol, mask_id)
            assert int(k_star[0]) == o_k and (accepted.cpu().numpy()[0] == o_acc).all()
            assert (d_x.cpu().numpy()[0] == x2).all()
            # the same acceptance on the oracle's own verifier tables: every per-position verdict that differs must
            # sit on a top-1 near-tie of that row or on a near pair of the parent's confidence ranking
            ov_top1, ov_conf = np.stack([t[0] for t in o_tabs]), np.stack([t[1] for t in o_tabs])
            spec = sorted({int(j) for j in o_sigma[:min(o_m, n_ranks)]})

            def committed(tabs_conf):
                return lambda p: set(orc.policy_select(orc.masked_in_block(o_drafts[p], bs, L, mask_id), tabs_conf[p], opol))

            v_g = G.edge_verdicts(v_top1_h, g_top1_h[0], spec, committed(v_conf_h))
            v_o = G.edge_verdicts(ov_top1, g_top1_h[0], spec, committed(ov_conf))
            for p, a in zip(*np.nonzero(v_g != v_o)):
                j = spec[a]
                if o_drafts[p][bs + j] != mask_id:
                    continue                      # p itself already holds position j: not an edge test
                tie_top1 = o_tabs[p][3][j] < 2 * eps_logit
                T_go, T_oo = committed(v_conf_h)(p), committed(ov_conf)(p)
                swapped = not G.unexplained_commit_differences(ov_conf[p], sorted(T_oo), sorted(T_go), opol.tau, r_conf)
                log["verdicts_differ"] += 1
                if not (tie_top1 or (T_go != T_oo and swapped)):
                    log["unexplained"] += 1
                    raise AssertionError(f"acceptance verdict of parent {p} at position {j} differs from the oracle's without a near-tie")
            if (v_g == v_o).all():
                o_acc2, o_k2 = orc.hierarchical_accept(o_drafts, bs, L, o_sigma, o_m, ograph, opol, ov_top1, ov_conf, mask_id)
                assert o_k2 == o_k and (o_acc2 == o_acc).all(), "same verdicts, different acceptance"
            x = x2
    return log


def test_config2_lockstep_first_blocks():
    w = inp.WORKLOADS[2]
    log = _lockstep(w, w.shape, n_blocks=2)
    print(f"[decode] config 2 lock-step: {log}", flush=True)
    assert log["iters"] >= 10


def test_config2_sharpened_head_lockstep():
    """Same model with logit_scale raised so that the threshold clause of the policy fires and drafts
    are accepted at depth (random-init logits are otherwise flat: confidences ~ 1e-3)."""
    import dataclasses
    w = inp.WORKLOADS[2]
    shape = dataclasses.replace(w.shape, logit_scale=11.0)
    log = _lockstep(w, shape, n_blocks=2, guard=11e-3)
    print(f"[decode] config 2 sharpened lock-step: {log}", flush=True)
    assert log["iters"] >= 4


def test_config3_width_two_layers_lockstep():
    """Config 3's widths, vocabulary, sequence and batch-of-drafts shape (4 x 512 tokens, d = 4096,
    V = 126464) with the depth cut to 2 layers so that the fp64 oracle keeps up; a few iterations."""
    w = inp.WORKLOADS[3]
    shape = inp.cut_down(w.shape, n_layers=2)
    log = _lockstep(w, shape, n_blocks=1, max_iters=3)
    print(f"[decode] config 3 (2 layers) lock-step: {log}", flush=True)
    assert log["iters"] == 3


def test_config4_shape_two_layers_lockstep():
    """Config 4's layout (grouped KV heads 28/4, QKV bias, d = 3584, F = 18944, V = 152064, N = 1024, K = 6)
    with the depth cut to 2 layers; two iterations against the oracle."""
    w = inp.WORKLOADS[4]
    shape = inp.cut_down(w.shape, n_layers=2)
    log = _lockstep(w, shape, n_blocks=1, max_iters=2)
    print(f"[decode] config 4 (2 layers) lock-step: {log}", flush=True)
    assert log["iters"] == 2


def test_config5_shape_batched_block_decode():
    """Config 5's batch shape (16 sequences of 1280 tokens, L = 64, K = 8: a verify call of 128 x 1280
    tokens) on a 2-layer cut of the model: one block through psd_decode_block and the loop invariants;
    then the model call for two of the sequences alone against the batched call."""
    import paper_2605_15609_amd as psd
    from paper_2605_15609_amd.synthetic import synthetic_model
    w = inp.WORKLOADS[5]
    shape = inp.cut_down(w.shape, n_layers=2, logit_scale=9.0)
    model = synthetic_model(shape, w.seq_len, DEV, threads=16)
    policy, graph = psd.Policy(w.tau, w.k_min, w.k_max), psd.chain_graph(w.n_drafts)
    tokens0 = inp.initial_state(w)
    together = _dev(tokens0)
    stats = psd.psd_decode_block(model, together, w.prompt_len, w.block_len, policy, graph)
    torch.cuda.synchronize()
    blk = together[:, w.prompt_len: w.prompt_len + w.block_len]
    assert not bool((blk == shape.mask_id).any())
    assert bool((together[:, w.prompt_len + w.block_len:] == shape.mask_id).all())      # later blocks untouched
    assert (together[:, : w.prompt_len].cpu().numpy() == tokens0[:, : w.prompt_len]).all()
    for s in stats:
        assert s.tokens == w.block_len and 1 <= s.invocations <= w.block_len and s.tpf >= 1.0
    print(f"[decode] config 5 shape: TPF per sequence {[round(s.tpf, 2) for s in stats]}", flush=True)
    # Batching changes which LM-head kernel runs (1024 rows: tiled; 64 rows: streaming), i.e. the order in
    # which the softmax normaliser is summed; confidences agree to fp32 rounding, tokens exactly.
    state = _dev(tokens0)
    t_all, c_all = psd.psd_forward_confidence(model, state, w.prompt_len, w.block_len)
    for b in (0, 11):
        t1, c1 = psd.psd_forward_confidence(model, _dev(tokens0[b: b + 1]), w.prompt_len, w.block_len)
        assert (t1[0] == t_all[b]).all(), b
        assert torch.allclose(c1[0], c_all[b], rtol=2e-6, atol=0), b


def test_config5_shape_two_layers_lockstep_inside_the_batch():
    """Config 5's launch shapes (16 x 1280 stage-1, 128 x 1280 verification, L = 64, K = 8) on a 2-layer cut: one
    iteration through the batched step calls.  The oracle's forward runs on sequences of the batch (one for the
    stage-1 tables; the root, one middle and the deepest draft of it for the verification tables); the decisions of
    all 16 sequences are replayed through the oracle's decision functions on the GPU's tables, bit for bit."""
    import paper_2605_15609_amd as psd
    from tests.gpu_common import gpu_graph
    w = inp.WORKLOADS[5]
    shape = inp.cut_down(w.shape, n_layers=2)
    N, bs, L, K, B = w.seq_len, w.prompt_len, w.block_len, w.n_drafts, w.batch
    host = inp.draw_model(shape, N, threads=16)
    model = psd.Model.from_host(host, DEV)
    opol, ograph = orc.Policy(w.tau, w.k_min, w.k_max), orc.chain_graph(K)
    gpol, ggraph = psd.Policy(w.tau, w.k_min, w.k_max), gpu_graph(ograph)
    mask_id = shape.mask_id
    x = inp.initial_state(w)
    log = {"near_tie_top1": 0, "max_conf_rel": 0.0, "unexplained": 0}
    eps_logit = 2e-2
    r_conf = float(np.expm1(2 * eps_logit))
    pick = 5
    d_x = _dev(x)
    g_top1, g_conf = psd.psd_forward_confidence(model, d_x, bs, L)
    t1, cf = g_top1.cpu().numpy(), g_conf.cpu().numpy()
    (o_top1, o_conf, _, _), = _check_tables(host, [x[pick]], bs, L, t1[pick:pick + 1], cf[pick:pick + 1], log, 1e-3, eps_logit)
    tm, ns = psd.psd_select_unmask(model, d_x, bs, L, g_top1, g_conf, gpol)
    sigma, m, drafts = psd.psd_build_drafts(model, d_x, bs, L, g_top1, g_conf, ggraph)
    after, sigma_h, m_h, drafts_h = d_x.cpu().numpy(), sigma.cpu().numpy(), m.cpu().numpy(), drafts.cpu().numpy()
    o_sig, o_m, o_dr = [None] * B, [0] * B, [None] * B
    for b in range(B):
        x1, _ = orc.select_unmask(x[b], bs, L, t1[b], cf[b], opol, mask_id)
        assert (after[b] == x1).all(), b
        o_sig[b], o_m[b], o_dr[b] = orc.build_drafts(x1, bs, L, t1[b], cf[b], ograph, mask_id)
        assert int(m_h[b]) == o_m[b] and (sigma_h[b] == o_sig[b]).all() and (drafts_h[b] == o_dr[b]).all(), b
    # the oracle on its own stage-1 tables of the picked sequence: only near pairs may differ
    x1_o, _ = orc.select_unmask(x[pick], bs, L, o_top1, o_conf, opol, mask_id)
    T_g = [j for j in range(L) if after[pick][bs + j] != mask_id]
    T_o = [j for j in range(L) if x1_o[bs + j] != mask_id]
    bad = G.unexplained_commit_differences(o_conf, T_o, T_g, opol.tau, r_conf)
    if set(T_o) == set(T_g):
        s_o, m_o, _ = orc.build_drafts(x1_o, bs, L, o_top1, o_conf, ograph, mask_id)
        bad += G.unexplained_rank_differences(o_conf, s_o[:m_o], o_sig[pick][:o_m[pick]], K - 1, r_conf)
    assert not bad, bad
    k_star, accepted, v_top1, v_conf = psd.psd_verify_accept(model, d_x, drafts, bs, L, sigma, m, ggraph, gpol)
    vt, vc = v_top1.cpu().numpy(), v_conf.cpu().numpy()
    nodes = [0, K // 2, K - 1]
    _check_tables(host, [o_dr[pick][k] for k in nodes], bs, L, vt[pick][nodes], vc[pick][nodes], log, 1e-3, eps_logit)
    final, ks_h, acc_h = d_x.cpu().numpy(), k_star.cpu().numpy(), accepted.cpu().numpy()
    for b in range(B):
        o_acc, o_k = orc.hierarchical_accept(o_dr[b], bs, L, o_sig[b], o_m[b], ograph, opol, vt[b], vc[b], mask_id)
        x2, _ = orc.advance(o_dr[b], o_k, bs, L, vt[b], vc[b], opol, mask_id)
        assert int(ks_h[b]) == o_k and (acc_h[b] == o_acc).all() and (final[b] == x2).all(), b
    print(f"[decode] config 5 shape (2 layers) lock-step inside the batch: {log}", flush=True)


def test_psd_decode_walks_every_sequence_through_its_own_blocks_like_the_oracle():
    """The whole generation behind one C call, fp32 model, exact: three sequences with prompts of different lengths start on
    different blocks and move on independently; tokens and counters of each must equal the oracle's decode of that sequence
    alone (also with EOS early stopping), and a run cut into single iterations must give the same result."""
    import paper_2605_15609_amd as psd
    shape = inp.WORKLOADS[1].shape
    N, L, B = 64, 16, 3
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    fn = orc.model_confidence_fn(host)
    prompts = (16, 32, 48)
    tokens0 = np.full((B, N), shape.mask_id, dtype=np.int32)
    for b, P in enumerate(prompts):
        tokens0[b, :P] = inp.draw_prompt(shape.vocab, P, 700 + b, "uniform")
    for K, tau in ((2, 0.9), (4, 0.02), (3, float("inf"))):
        refs = [orc.decode(fn, tokens0[b], prompts[b], L, orc.Policy(tau, 1, 0), orc.chain_graph(K), shape.mask_id) for b in range(B)]
        d = _dev(tokens0)
        stats, starts, iters = psd.psd_decode(model, d, list(prompts), L, psd.Policy(tau, 1, 0), psd.chain_graph(K))
        got = d.cpu().numpy()
        assert all(s >= N for s in starts) and iters >= 1
        for b in range(B):
            assert (got[b] == refs[b][0]).all(), (K, tau, b)
            assert _counters(stats[b]) == _counters(refs[b][1]), (K, tau, b)
        # the same generation, one iteration of the batch per call
        d1 = _dev(tokens0)
        st, at, total = None, list(prompts), 0
        for _ in range(10 * N):
            st, at, n = psd.psd_decode(model, d1, at, L, psd.Policy(tau, 1, 0), psd.chain_graph(K), st, max_iterations=1)
            total += n
            if n == 0:
                break
        assert (d1.cpu().numpy() == got).all() and total == iters, (K, tau)
        assert [_counters(s) for s in st] == [_counters(s) for s in stats]
        # EOS early stopping: a token the free run of sequence 0 produces in its second block
        eos = int(refs[0][0][prompts[0] + L + 3])
        d2 = _dev(tokens0)
        stats2, starts2, _ = psd.psd_decode(model, d2, list(prompts), L, psd.Policy(tau, 1, 0, eos_id=eos), psd.chain_graph(K))
        for b in range(B):
            ref, ost = orc.decode(fn, tokens0[b], prompts[b], L, orc.Policy(tau, 1, 0), orc.chain_graph(K), shape.mask_id, eos_id=eos)
            assert (d2.cpu().numpy()[b] == ref).all(), (K, tau, b, "eos")
            assert _counters(stats2[b]) == _counters(ost), (K, tau, b, "eos")
        assert stats2[0].stopped
    with pytest.raises(psd.PsdError):
        psd.psd_decode(model, _dev(tokens0), [16, 30, 48], L, psd.Policy(), psd.chain_graph(2))     # not whole blocks


def test_single_forward_loop_matches_the_oracle_variant_sequence_by_sequence():
    """policy.single_forward: one model call per iteration -- the post-verification commit is the next stage-1 commit and the
    next drafts come from the accepted draft's verifier output.  fp32 model, exact: three sequences on blocks of their own in
    one batch; tokens and every counter must equal the oracle's single-forward decode of each sequence alone, for chains and
    a subset lattice, with and without EOS early stopping; the calls saved against the literal loop are counted."""
    import paper_2605_15609_amd as psd
    from tests.gpu_common import gpu_graph
    shape = inp.WORKLOADS[1].shape
    N, L, B = 64, 16, 3
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    fn = orc.model_confidence_fn(host)
    prompts = (16, 32, 48)
    tokens0 = np.full((B, N), shape.mask_id, dtype=np.int32)
    for b, P in enumerate(prompts):
        tokens0[b, :P] = inp.draw_prompt(shape.vocab, P, 700 + b, "uniform")
    differs = 0
    for ograph, tau, k_max in ((orc.chain_graph(2), 0.9, 0), (orc.chain_graph(4), 0.02, 0), (orc.chain_graph(3), float("inf"), 0),
                               (orc.Graph((frozenset(), frozenset({0}), frozenset({1}), frozenset({0, 1}))), 0.05, 0), (orc.chain_graph(4), 0.02, 2)):
        opol, ggraph = orc.Policy(tau, 1, k_max), gpu_graph(ograph)
        refs = [orc.decode(fn, tokens0[b], prompts[b], L, opol, ograph, shape.mask_id, single_forward=True) for b in range(B)]
        literal = [orc.decode(fn, tokens0[b], prompts[b], L, opol, ograph, shape.mask_id) for b in range(B)]
        d = _dev(tokens0)
        stats, starts, iters = psd.psd_decode(model, d, list(prompts), L, psd.Policy(tau, 1, k_max, single_forward=True), ggraph)
        got = d.cpu().numpy()
        assert all(s >= N for s in starts)
        for b in range(B):
            assert (got[b] == refs[b][0]).all(), (ograph.K, tau, b)
            assert _counters(stats[b]) == _counters(refs[b][1]), (ograph.K, tau, b)
            n_blocks = (N - prompts[b]) // L
            # one stage-1 call per block entered, every other call is a batched verification
            assert stats[b].invocations == n_blocks + sum(stats[b].depth_hist), (ograph.K, tau, b)
            assert stats[b].invocations <= literal[b][1].invocations or not (got[b] == literal[b][0]).all()
            differs += int(not (got[b] == literal[b][0]).all())
        # the literal loop through the same entry point is untouched by the flag being there
        d0 = _dev(tokens0)
        st0, _, _ = psd.psd_decode(model, d0, list(prompts), L, psd.Policy(tau, 1, k_max), ggraph)
        for b in range(B):
            assert (d0.cpu().numpy()[b] == literal[b][0]).all() and _counters(st0[b]) == _counters(literal[b][1])
        # EOS early stopping: a token the single-forward run of sequence 0 produces in its second block
        eos = int(refs[0][0][prompts[0] + L + 3])
        d2 = _dev(tokens0)
        stats2, _, _ = psd.psd_decode(model, d2, list(prompts), L, psd.Policy(tau, 1, k_max, eos_id=eos, single_forward=True), ggraph)
        for b in range(B):
            ref, ost = orc.decode(fn, tokens0[b], prompts[b], L, opol, ograph, shape.mask_id, eos_id=eos, single_forward=True)
            assert (d2.cpu().numpy()[b] == ref).all(), (ograph.K, tau, b, "eos")
            assert _counters(stats2[b]) == _counters(ost), (ograph.K, tau, b, "eos")
        assert stats2[0].stopped
    print(f"[decode] single-forward loop: {differs} of {5 * B} generations differ from the literal loop's", flush=True)
    # one block through psd_decode_block, every sequence on its own start
    d = _dev(tokens0)
    stats = psd.psd_decode_block(model, d, list(prompts), L, psd.Policy(0.9, 1, 0, single_forward=True), psd.chain_graph(3))
    for b in range(B):
        ref, ost = orc.decode_block(fn, tokens0[b], prompts[b], L, orc.Policy(0.9, 1, 0), orc.chain_graph(3), shape.mask_id,
                                    single_forward=True)
        assert (d.cpu().numpy()[b] == ref).all() and _counters(stats[b]) == _counters(ost), b


def test_single_forward_loop_bf16_batch_equals_sequences_alone():
    import paper_2605_15609_amd as psd
    shape = inp.cut_down(inp.WORKLOADS[2].shape, n_layers=2, vocab=4000, seed=33, logit_scale=14.0)
    N, L, K, B = 160, 32, 4, 4
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    policy, graph = psd.Policy(0.9, 1, 0, single_forward=True), psd.chain_graph(K)
    starts = [64, 96, 32, 64]
    tokens = np.full((B, N), shape.mask_id, dtype=np.int32)
    for b in range(B):
        tokens[b, :starts[b]] = inp.draw_prompt(shape.vocab, starts[b], 80 + b)
    together = _dev(tokens)
    stats, at, _ = psd.psd_decode(model, together, starts, L, policy, graph)
    saved = 0
    for b in range(B):
        alone = _dev(tokens[b: b + 1])
        s, _, _ = psd.psd_decode(model, alone, [starts[b]], L, policy, graph)
        assert (alone[0] == together[b]).all(), b
        assert _counters(s[0]) == _counters(stats[b]), b
        assert (together[b] != shape.mask_id).all() and stats[b].tokens == N - starts[b]
        lit = _dev(tokens[b: b + 1])
        s_lit, _, _ = psd.psd_decode(model, lit, [starts[b]], L, psd.Policy(0.9, 1, 0), graph)
        saved += s_lit[0].invocations - s[0].invocations
    print(f"[decode] single-forward loop, bf16: {saved} model calls fewer than the literal loop over {B} sequences", flush=True)


def test_model_calls_replayed_as_hip_graphs_give_the_same_generation():
    """Optional HIP-graph replay of the block loop's model calls: a call seen twice is captured, then replayed.  Every
    replay must leave what the eager launches leave: whole generations with graphs on equal those with graphs off, run
    alternately (eager work and synchronisations between the replays), over several distinct batches so that a graph is
    replayed on token contents it was not captured with."""
    import paper_2605_15609_amd as psd
    shape = inp.cut_down(inp.WORKLOADS[2].shape, n_layers=2, vocab=4000, seed=33, logit_scale=14.0)
    N, L, K, B = 160, 32, 3, 3
    model = psd.Model.from_host(inp.draw_model(shape, N), DEV)
    policy, graph = psd.Policy(0.9, 1, 0), psd.chain_graph(K)
    replays = 0
    d = torch.empty((B, N), dtype=torch.int32, device=DEV)      # one buffer: the graphs hold its address
    for round_ in range(3):
        tokens = np.full((B, N), shape.mask_id, dtype=np.int32)
        for b in range(B):
            tokens[b, :64] = inp.draw_prompt(shape.vocab, 64, 500 + 10 * round_ + b)
        results = []
        for on in (False, True):
            model.set_graphs(on)
            d.copy_(torch.from_numpy(tokens))
            stats, _, iters = psd.psd_decode(model, d, 64, L, policy, graph)
            results.append((d.cpu().numpy(), [_counters(s) for s in stats], iters))
        assert (results[0][0] == results[1][0]).all() and results[0][1:] == results[1][1:], round_
        assert (results[1][0] != shape.mask_id).all()
        now = model.set_graphs(False)
        assert now > replays, "the graph path did not run"
        replays = now
    print(f"[decode] {replays} model calls replayed from HIP graphs", flush=True)


def test_psd_decode_block_with_one_block_start_per_sequence():
    import paper_2605_15609_amd as psd
    shape = inp.cut_down(inp.WORKLOADS[2].shape, n_layers=2, vocab=4000, seed=33, logit_scale=14.0)
    N, L, K, B = 160, 32, 3, 4
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    policy, graph = psd.Policy(0.9, 1, 0), psd.chain_graph(K)
    starts = [64, 96, 32, 64]
    tokens = np.full((B, N), shape.mask_id, dtype=np.int32)
    for b in range(B):
        tokens[b, :starts[b]] = inp.draw_prompt(shape.vocab, starts[b], 80 + b)
    together = _dev(tokens)
    stats = psd.psd_decode_block(model, together, starts, L, policy, graph)
    for b in range(B):
        alone = _dev(tokens[b: b + 1])
        s = psd.psd_decode_block(model, alone, starts[b], L, policy, graph)
        assert (alone[0] == together[b]).all(), b
        assert (s[0].invocations, s[0].tokens) == (stats[b].invocations, stats[b].tokens) and s[0].tokens == L
        row = together[b].cpu().numpy()
        assert (row[starts[b]: starts[b] + L] != shape.mask_id).all() and (row[starts[b] + L:] == shape.mask_id).all()
