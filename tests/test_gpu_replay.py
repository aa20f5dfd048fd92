"""Decision parity at the full size of the 7-8B-parameter configurations (full depth, width, vocabulary, batch), with
no exclusions: the real HIP decode runs through the step calls of the C ABI, and at every iteration the tables the GPU
model produced -- (top1, conf) of the stage-1 call and of the batched verification call -- go through the oracle's
decision functions (policy and Eq. 1, speculative ordering and Eq. 2, hierarchical acceptance, advance).  The committed
positions, sigma, m, every draft, the accepted set, k* and the new state must be bit-identical for every sequence at
every iteration.  No oracle forward is needed, so this covers what a lock-step against the fp64 forward cannot afford:
configs 3 and 4 over whole blocks at 32 / 28 layers and config 5 with all 16 sequences in the 16 x 1280 and 128 x 1280
launch shapes the benchmark times.  The same trajectory must also come out of psd_decode_block."""
import numpy as np
import pytest
import torch

import psd_inputs as inp
from oracle import psd_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _valid_tables(block_tokens, top1, conf, mask_id, where):
    """Model outputs must be predictions: a vocabulary token other than [M] with a confidence in (0, 1] on every masked
    position, the sentinel (own token, -1) elsewhere."""
    masked = block_tokens == mask_id
    assert np.isfinite(conf).all(), where
    assert ((conf[masked] > 0) & (conf[masked] <= 1)).all(), where
    assert ((top1[masked] >= 0) & (top1[masked] < mask_id)).all(), where
    assert (top1[~masked] == block_tokens[~masked]).all() and (conf[~masked] == -1).all(), where


def _replay(cfg, n_blocks, max_iters_per_block=10 ** 9, check_decode_block=True):
    import paper_2605_15609_amd as psd
    from paper_2605_15609_amd.synthetic import synthetic_model
    from tests.gpu_common import gpu_graph, say
    w = inp.WORKLOADS[cfg]
    shape, N, P, L, K, B = w.shape, w.seq_len, w.prompt_len, w.block_len, w.n_drafts, w.batch
    model = synthetic_model(shape, N, DEV, threads=16)
    opol, ograph = orc.Policy(w.tau, w.k_min, w.k_max), orc.chain_graph(K)
    gpol, ggraph = psd.Policy(w.tau, w.k_min, w.k_max), gpu_graph(ograph)
    mask_id = shape.mask_id
    tokens0 = inp.initial_state(w)
    d_x = torch.from_numpy(tokens0).to(DEV)
    x = tokens0.copy()                      # the oracle's copy of the state, advanced by the oracle's decisions
    log = {"iterations": 0, "sequence_iterations": 0, "verify_calls": 0, "tokens": 0, "depth_hist": [0] * K}
    invocations = np.zeros(B, dtype=np.int64)
    for blk in range(n_blocks):
        bs = P + blk * L
        it = 0
        while (x[:, bs: bs + L] == mask_id).any() and it < max_iters_per_block:
            it += 1
            log["iterations"] += 1
            live = [b for b in range(B) if (x[b, bs: bs + L] == mask_id).any()]
            g_top1, g_conf = psd.psd_forward_confidence(model, d_x, bs, L)            # stage 1, the whole batch
            t1, cf = g_top1.cpu().numpy(), g_conf.cpu().numpy()
            _valid_tables(x[:, bs: bs + L], t1, cf, mask_id, (cfg, blk, it, "stage-1 tables"))
            tm, ns = psd.psd_select_unmask(model, d_x, bs, L, g_top1, g_conf, gpol)
            sigma, m, drafts = psd.psd_build_drafts(model, d_x, bs, L, g_top1, g_conf, ggraph)
            after_commit, tm_h = d_x.cpu().numpy(), tm.cpu().numpy()
            sigma_h, m_h, drafts_h = sigma.cpu().numpy(), m.cpu().numpy(), drafts.cpu().numpy()
            o_sig, o_m, o_dr = [None] * B, np.zeros(B, dtype=np.int64), [None] * B
            for b in range(B):
                x1, o_tm = orc.select_unmask(x[b], bs, L, t1[b], cf[b], opol, mask_id)
                assert (after_commit[b] == x1).all() and (tm_h[b] == o_tm).all(), (cfg, blk, it, b, "stage-1 commit")
                o_sig[b], o_m[b], o_dr[b] = orc.build_drafts(x1, bs, L, t1[b], cf[b], ograph, mask_id)
                assert int(m_h[b]) == o_m[b] and (sigma_h[b] == o_sig[b]).all(), (cfg, blk, it, b, "sigma / m")
                assert (drafts_h[b] == o_dr[b]).all(), (cfg, blk, it, b, "drafts")
                x[b] = x1
                log["tokens"] += int(o_tm.sum())
            invocations[live] += 1
            log["sequence_iterations"] += len(live)
            if not (o_m > 0).any():
                continue
            k_star, accepted, v_top1, v_conf = psd.psd_verify_accept(model, d_x, drafts, bs, L, sigma, m, ggraph, gpol)
            log["verify_calls"] += 1
            vt, vc = v_top1.cpu().numpy(), v_conf.cpu().numpy()
            for b in range(B):
                if o_m[b] > 0:
                    _valid_tables(np.stack(o_dr[b])[:, bs: bs + L], vt[b], vc[b], mask_id, (cfg, blk, it, b, "verification tables"))
            after, ks_h, acc_h = d_x.cpu().numpy(), k_star.cpu().numpy(), accepted.cpu().numpy()
            for b in range(B):
                if o_m[b] == 0:
                    assert (after[b] == x[b]).all(), (cfg, blk, it, b, "a finished sequence was touched")
                    continue
                invocations[b] += 1
                o_acc, o_k = orc.hierarchical_accept(o_dr[b], bs, L, o_sig[b], int(o_m[b]), ograph, opol, vt[b], vc[b], mask_id)
                x2, n_post = orc.advance(o_dr[b], o_k, bs, L, vt[b], vc[b], opol, mask_id)
                assert int(ks_h[b]) == o_k and (acc_h[b] == o_acc).all(), (cfg, blk, it, b, "acceptance")
                assert (after[b] == x2).all(), (cfg, blk, it, b, "advance")
                depth = len(orc.node_positions(ograph, [int(s) for s in o_sig[b][:o_m[b]]])[o_k])
                log["depth_hist"][depth] += 1
                log["tokens"] += depth + n_post
                x[b] = x2
        say(f"[replay] config {cfg} block {blk}: {log}")
    if check_decode_block:
        # the block loop of the library must walk the very same trajectory
        d_y = torch.from_numpy(tokens0).to(DEV)
        stats = None
        for blk in range(n_blocks):
            stats = psd.psd_decode_block(model, d_y, P + blk * L, L, gpol, ggraph, stats)
        assert (d_y.cpu().numpy() == x).all(), "psd_decode_block left the trajectory of the step calls"
        assert [s.invocations for s in stats] == invocations.tolist()
        assert sum(s.tokens for s in stats) == log["tokens"]
    model.close()
    return log


def test_config3_full_depth_two_blocks_every_decision_replayed():
    log = _replay(3, n_blocks=2)
    assert log["tokens"] == 2 * 32 and log["verify_calls"] >= 8


def test_config4_full_depth_first_block_every_decision_replayed():
    log = _replay(4, n_blocks=1)
    assert log["tokens"] == 32 and log["verify_calls"] >= 4


def test_config5_full_depth_first_block_all_sixteen_sequences_replayed():
    """16 x 1280 stage-1 calls and 128 x 1280 verification calls at 32 layers: about a minute of GPU time."""
    log = _replay(5, n_blocks=1, check_decode_block=False)
    assert log["tokens"] == 16 * 64 and log["sequence_iterations"] >= 16 * 8
