"""Bit-exact parity of the HIP decision kernels (select_unmask, build_drafts, accept) with
the oracle on identical fp32 (top1, conf) tables, through the C ABI."""
import numpy as np
import pytest
import torch

import psd_inputs as inp
from oracle import psd_oracle as orc

pytestmark = pytest.mark.gpu

INF = float("inf")


@pytest.fixture(scope="module")
def env():
    import paper_2605_15609_amd as psd
    from tests.gpu_common import make_models
    shape = inp.cut_down(inp.WORKLOADS[1].shape, n_layers=1, vocab=1000, seed=77)
    host, model = make_models(shape, 2048)
    return psd, model


CASES = [
    # B, N, block_start, L, K, width, tau, k_min, k_max, conf_kind, ties
    (1, 48, 16, 32, 2, 1, 0.9, 1, 0, "uniform", 0),
    (3, 20, 5, 7, 3, 1, 0.5, 1, 0, "uniform", 0),
    (4, 70, 6, 64, 5, 2, 0.9, 1, 0, "uniform", 4),
    (5, 384, 128, 32, 4, 1, 0.9, 1, 0, "low", 0),
    (2, 512, 256, 32, 4, 1, INF, 1, 0, "uniform", 0),
    (2, 512, 480, 32, 4, 1, 0.3, 2, 5, "uniform", 3),
    (16, 1280, 256, 64, 8, 1, 0.9, 1, 0, "uniform", 0),
    (16, 1280, 1216, 64, 8, 1, 0.9, 1, 0, "high", 0),
    (2, 1024, 512, 32, 6, 1, 0.9, 1, 0, "uniform", 0),
    (2, 64, 0, 1, 2, 1, 0.9, 1, 0, "uniform", 0),
    (3, 200, 100, 33, 32, 1, 0.7, 0, 0, "uniform", 5),
]


@pytest.mark.parametrize("case", CASES, ids=[f"B{c[0]}-N{c[1]}-L{c[3]}-K{c[4]}-{c[9]}" for c in CASES])
def test_decision_kernels_match_oracle_bit_exactly(env, case):
    psd, model = env
    from tests.gpu_common import to_dev, gpu_graph, say
    B, N, bs, L, K, width, tau, k_min, k_max, kind, ties = case
    vocab, mask_id = model.shape.vocab, model.shape.mask_id
    say(f"[decisions] case {case}")
    for rep in range(6):
        frac = [0.0, 0.15, 0.5, 0.8, 1.0, 0.95][rep]
        toks, top1s, confs = zip(*[inp.draw_block_state(1000 * rep + b, N, bs, L, vocab, frac_masked=frac, conf_kind=kind,
                                                        tie_levels=ties) for b in range(B)])
        tokens, top1, conf = np.stack(toks), np.stack(top1s), np.stack(confs)
        ograph = orc.chain_graph(K, width)
        opol = orc.Policy(tau, k_min, k_max)
        gpol, ggraph = psd.Policy(tau, k_min, k_max), gpu_graph(ograph)

        d_tokens, d_top1, d_conf = to_dev(tokens), to_dev(top1), to_dev(conf)
        tm, ns = psd.psd_select_unmask(model, d_tokens, bs, L, d_top1, d_conf, gpol)
        sigma, m, drafts = psd.psd_build_drafts(model, d_tokens, bs, L, d_top1, d_conf, ggraph)
        x1 = d_tokens.cpu().numpy()
        drafts_h = drafts.cpu().numpy()
        v = [inp.draw_verifier_tables(5000 * rep + b, drafts_h[b], bs, L, vocab, top1[b], agree=0.8, conf_kind=kind)
             for b in range(B)]
        v_top1, v_conf = np.stack([a for a, _ in v]), np.stack([c for _, c in v])
        k_star, accepted = psd.psd_accept(model, d_tokens, drafts, bs, L, sigma, m, ggraph, gpol, to_dev(v_top1),
                                          to_dev(v_conf))
        torch.cuda.synchronize()
        x2 = d_tokens.cpu().numpy()
        tm, ns, sigma, m, k_star, accepted = (t.cpu().numpy() for t in (tm, ns, sigma, m, k_star, accepted))

        for b in range(B):
            o_x1, o_tm = orc.select_unmask(tokens[b], bs, L, top1[b], conf[b], opol, mask_id)
            assert (x1[b] == o_x1).all() and (tm[b] == o_tm).all() and ns[b] == o_tm.sum()
            o_sigma, o_m, o_drafts = orc.build_drafts(o_x1, bs, L, top1[b], conf[b], ograph, mask_id)
            assert m[b] == o_m and (sigma[b] == o_sigma).all() and (drafts_h[b] == o_drafts).all()
            if o_m == 0:
                assert k_star[b] == 0 and (x2[b] == o_x1).all()
                continue
            o_acc, o_k = orc.hierarchical_accept(o_drafts, bs, L, o_sigma, o_m, ograph, opol, v_top1[b], v_conf[b], mask_id)
            o_x2, _ = orc.advance(o_drafts, o_k, bs, L, v_top1[b], v_conf[b], opol, mask_id)
            assert k_star[b] == o_k and (accepted[b] == o_acc).all()
            assert (x2[b] == o_x2).all()


def test_random_dags_match_oracle(env):
    psd, model = env
    from tests.gpu_common import to_dev, gpu_graph
    vocab, mask_id = model.shape.vocab, model.shape.mask_id
    rng = np.random.default_rng(3)
    depths = set()
    for trial in range(40):
        L = int(rng.integers(4, 40))
        K = int(rng.integers(2, 12))
        N, bs = L + 9, 4
        sets = {frozenset()}
        while len(sets) < K:
            size = int(rng.integers(1, 6))
            sets.add(frozenset(int(r) for r in rng.choice(8, size=size, replace=False)))
        ograph = orc.Graph(tuple(sorted(sets, key=lambda s: (len(s), sorted(s)))))
        opol = orc.Policy(float(rng.choice([0.0, 0.5, 0.9])), int(rng.integers(0, 3)), 0)
        gpol, ggraph = psd.Policy(opol.tau, opol.k_min, 0), gpu_graph(ograph)
        tokens, top1, conf = inp.draw_block_state(trial, N, bs, L, vocab, frac_masked=0.9)
        x1, _ = orc.select_unmask(tokens, bs, L, top1, conf, orc.Policy(INF, 1), mask_id)
        o_sigma, o_m, o_drafts = orc.build_drafts(x1, bs, L, top1, conf, ograph, mask_id)
        d_x1 = to_dev(x1[None])
        sigma, m, drafts = psd.psd_build_drafts(model, d_x1, bs, L, to_dev(top1[None]), to_dev(conf[None]), ggraph)
        assert (drafts[0].cpu().numpy() == o_drafts).all() and int(m[0]) == o_m
        v_top1, v_conf = inp.draw_verifier_tables(trial + 99, o_drafts, bs, L, vocab, top1, agree=0.9)
        k_star, accepted = psd.psd_accept(model, d_x1, drafts, bs, L, sigma, m, ggraph, gpol, to_dev(v_top1[None]),
                                          to_dev(v_conf[None]))
        o_acc, o_k = orc.hierarchical_accept(o_drafts, bs, L, o_sigma, o_m, ograph, opol, v_top1, v_conf, mask_id)
        o_x2, _ = orc.advance(o_drafts, o_k, bs, L, v_top1, v_conf, opol, mask_id)
        assert int(k_star[0]) == o_k and (accepted[0].cpu().numpy() == o_acc).all()
        assert (d_x1[0].cpu().numpy() == o_x2).all()
        depths.add(len(orc.node_positions(ograph, [int(s) for s in o_sigma[:o_m]])[o_k]))
    assert len(depths) >= 3


def test_argument_errors_are_reported_not_launched(env):
    psd, model = env
    from tests.gpu_common import to_dev
    tokens = to_dev(np.zeros((1, 32), dtype=np.int32))
    top1 = to_dev(np.zeros((1, 65), dtype=np.int32))
    conf = to_dev(np.zeros((1, 65), dtype=np.float32))
    with pytest.raises(psd.PsdError, match="block length"):
        psd.psd_select_unmask(model, tokens, 0, 65, top1, conf, psd.Policy())
    with pytest.raises(psd.PsdError, match="outside the sequence"):
        psd.psd_select_unmask(model, tokens, 20, 16, top1, conf, psd.Policy())
    with pytest.raises(psd.PsdError, match="root"):
        psd.psd_build_drafts(model, tokens, 0, 16, top1, conf, psd.Graph((1, 3)))
    with pytest.raises(psd.PsdError):
        psd.psd_select_unmask(model, tokens, 0, 16, top1, conf, psd.Policy(tau=float("nan")))
    # EOS early stopping needs a token id other than the mask token
    for bad in (model.cfg.mask_id, model.cfg.vocab, -3):
        with pytest.raises(psd.PsdError, match="eos_id"):
            psd.psd_decode_block(model, tokens, 0, 16, psd.Policy(eos_id=bad), psd.chain_graph(2))
