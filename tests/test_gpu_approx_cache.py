"""Approximate prefix + suffix KV cache for fully bidirectional models, against the oracle's ApproximateCache.

The mode changes results (stale context), so the reference is the oracle run in the same mode: the call that enters
a block is exact and freezes every layer's keys / values outside the block; later calls recompute the block rows
against them.  Checked: (1) refresh and cached calls, stage-1 shape and a verification batch whose drafts share
their sequence's cache, fp32 within 1e-4 and bf16 within 2e-2 of the oracle's logits, decisions as in the exact
tests; (2) the approximation is real (cached logits differ from the exact forward) yet the first call is the exact
one; (3) a free-running fp32 decode reproduces the oracle's decode under the same cache token for token;
(4) a batched bf16 decode equals the sequences decoded alone."""
import dataclasses

import numpy as np
import pytest
import torch

import psd_inputs as inp
from oracle import psd_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

FP32 = inp.cut_down(inp.WORKLOADS[4].shape, name="ac-fp32", dtype="fp32", n_layers=2, d_model=96, n_heads=6, n_kv_heads=2,
                    d_head=16, d_ffn=160, vocab=211, seed=51)
BF16 = {
    "mha-dh64": inp.cut_down(inp.WORKLOADS[2].shape, n_layers=2, vocab=5000, seed=52),
    "gqa-bias-dh128": inp.cut_down(inp.WORKLOADS[4].shape, n_layers=2, d_model=512, n_heads=4, n_kv_heads=2, d_ffn=640,
                                   vocab=3001, seed=53),
}


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _entry_state(shape, N, P, L, block, seed):
    """prompt, `block` finished generation blocks, the active block and everything behind it masked"""
    t = np.full(N, shape.mask_id, dtype=np.int32)
    start = P + block * L
    t[:start] = inp.draw_prompt(shape.vocab, start, seed)
    return t, start


def _check(ref_fn_out, z, shape, logits, top1, conf, t, start, L, tol, label):
    from tests.test_gpu_forward import check_sequence
    o_top1, o_conf = ref_fn_out
    return check_sequence((o_top1, o_conf, z, None), logits, top1, conf, t, shape.mask_id, start, L, tol, label)


def _steps(shape, P, L, G, block, tol, K=4):
    """refresh call, then a stage-1-shaped cached call and a verification batch after commits, vs the oracle's cache"""
    import paper_2605_15609_amd as psd
    N = P + G
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    t0, start = _entry_state(shape, N, P, L, block, 7)
    ocache = orc.ApproximateCache(host)
    cache = psd.KvCache(model, 1, N - L)
    # the call that enters the block: exact
    ref = ocache(t0, start, L)
    top1, conf, logits = psd.psd_forward_confidence_approx(model, _dev(t0[None]), start, L, cache, refresh=True, want_logits=True)
    _check(ref, ocache.logits, shape, logits.cpu().numpy(), top1[0].cpu().numpy(), conf[0].cpu().numpy(), t0, start, L, tol, "refresh")
    z_exact = orc.forward_confidence(host, t0, start, L, return_logits=True)[2]
    assert np.abs(ocache.logits - z_exact).max() < 1e-9
    # a few positions committed (the oracle's own predictions): block rows against the frozen context
    rng = np.random.default_rng(3)
    t1 = t0.copy()
    idx = rng.choice(L, size=5, replace=False)
    t1[start + idx] = ref[0][idx]
    ref1 = ocache(t1, start, L)
    z1 = ocache.logits.copy()
    top1, conf, logits = psd.psd_forward_confidence_approx(model, _dev(t1[None]), start, L, cache, refresh=False, want_logits=True)
    _check(ref1, z1, shape, logits.cpu().numpy(), top1[0].cpu().numpy(), conf[0].cpu().numpy(), t1, start, L, tol, "cached")
    stale = np.abs(z1 - orc.forward_confidence(host, t1, start, L, return_logits=True)[2]).max()
    assert stale > 10 * (1e-4 if shape.dtype == "fp32" else 1e-3)          # the approximation is visible
    # a verification batch: K drafts of the one sequence share its cache
    drafts = np.repeat(t1[None], K, axis=0)
    order = [j for j in range(L) if t1[start + j] == shape.mask_id]
    for k in range(1, K):
        for j in order[:k]:
            drafts[k, start + j] = ref1[0][j]
    top1, conf, logits = psd.psd_forward_confidence_approx(model, _dev(drafts), start, L, cache, refresh=False, seqs_per_cache=K,
                                                           want_logits=True)
    lg = logits.cpu().numpy().reshape(K, L, -1)
    for k in range(K):
        refk = ocache(drafts[k], start, L)
        _check(refk, ocache.logits, shape, lg[k], top1[k].cpu().numpy(), conf[k].cpu().numpy(), drafts[k], start, L, tol, f"draft {k}")


@pytest.mark.parametrize("L,block", [(16, 0), (32, 1), (64, 0)])
def test_fp32_refresh_and_cached_calls_match_the_oracle_cache(L, block):
    _steps(FP32, 2 * L - 8, L, 3 * L, block, 1e-4)          # a prompt that is not a multiple of the block length


@pytest.mark.parametrize("name", list(BF16))
def test_bf16_refresh_and_cached_calls_match_the_oracle_cache(name):
    _steps(BF16[name], 72, 32, 96, 1, 2e-2)


def test_fp32_free_running_decode_under_the_cache_matches_the_oracle():
    import paper_2605_15609_amd as psd
    shape = FP32
    L, P, G = 16, 24, 48
    N = P + G
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    differs = 0
    for K, tau in ((3, 0.9), (4, 0.05), (1, 0.9)):
        tokens0 = np.full((1, N), shape.mask_id, dtype=np.int32)
        tokens0[0, :P] = inp.draw_prompt(shape.vocab, P, 61)
        d = _dev(tokens0)
        cache = psd.KvCache(model, 1, N - L)
        stats = [psd.Stats()]
        for start in range(P, N, L):
            stats = psd.psd_decode_block_approx(model, d, start, L, psd.Policy(tau, 1, 0), psd.chain_graph(K), cache, stats)
        ocache = orc.ApproximateCache(host)
        ref, ost = orc.decode(ocache, tokens0[0], P, L, orc.Policy(tau, 1, 0), orc.chain_graph(K), shape.mask_id)
        assert (d.cpu().numpy()[0] == ref).all(), (K, tau)
        s = stats[0]
        assert (s.invocations, s.tokens_policy, s.tokens_draft, s.tokens_postverify) == \
               (ost.invocations, ost.tokens_policy, ost.tokens_draft, ost.tokens_postverify)
        assert s.depth_hist[:32] == ost.depth_hist and ocache.refreshes == G // L
        exact, _ = orc.decode(orc.model_confidence_fn(host), tokens0[0], P, L, orc.Policy(tau, 1, 0), orc.chain_graph(K),
                              shape.mask_id)
        differs += int((exact != ref).any())
    assert differs >= 1            # the cache does change the decode somewhere: this is not the exact path in disguise


def test_bf16_batched_decode_under_the_cache_equals_sequences_alone():
    import paper_2605_15609_amd as psd
    shape = dataclasses.replace(BF16["mha-dh64"], logit_scale=14.0)
    L, P, G, K, B = 32, 40, 64, 2, 2
    N = P + G
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    policy, graph = psd.Policy(0.9, 1, 0), psd.chain_graph(K)
    tokens = np.full((B, N), shape.mask_id, dtype=np.int32)
    for b in range(B):
        tokens[b, :P] = inp.draw_prompt(shape.vocab, P, 80 + b)

    def run(batch):
        d = _dev(batch)
        cache = psd.KvCache(model, batch.shape[0], N - L)
        stats = [psd.Stats() for _ in range(batch.shape[0])]
        for start in range(P, N, L):
            stats = psd.psd_decode_block_approx(model, d, start, L, policy, graph, cache, stats)
        return d.cpu().numpy(), stats

    together, st = run(tokens)
    assert not (together == shape.mask_id).any()
    for b in range(B):
        alone, s1 = run(tokens[b:b + 1])
        assert (alone[0] == together[b]).all(), b
        assert (s1[0].invocations, s1[0].tokens) == (st[b].invocations, st[b].tokens)
    assert all(s.tpf >= 1.0 for s in st)


def test_argument_errors():
    import paper_2605_15609_amd as psd
    shape = FP32
    N, L = 64, 16
    model = psd.Model.from_host(inp.draw_model(shape, N), DEV)
    d = _dev(np.full((1, N), shape.mask_id, dtype=np.int32))
    small = psd.KvCache(model, 1, N - L - 1)
    with pytest.raises(psd.PsdError):
        psd.psd_forward_confidence_approx(model, d, 16, L, small, refresh=True)              # cache too small
    cache = psd.KvCache(model, 1, N - L)
    with pytest.raises(psd.PsdError):
        psd.psd_forward_confidence_approx(model, d, 16, 8, cache, refresh=True)              # block length not a multiple of 16
    with pytest.raises(psd.PsdError):
        psd.psd_forward_confidence_approx(model, d.repeat(2, 1), 16, L, cache, refresh=True, seqs_per_cache=2)
    bc = psd.Model.from_host(inp.draw_model(dataclasses.replace(shape, attention="block_causal"), N), DEV)
    with pytest.raises(psd.PsdError):
        psd.psd_decode_block_approx(bc, d, 16, L, psd.Policy(), psd.chain_graph(2), psd.KvCache(bc, 1, N))   # exact cache exists
    with pytest.raises(psd.PsdError):
        psd.psd_kv_prefill(model, d, 16, L, cache)                                           # the exact cache calls need block-causal
