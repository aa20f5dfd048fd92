"""The 7B/8B-parameter configurations at their full size, in the launch configurations the benchmark times,
against the fp64 oracle over the full depth: config 3 (32 layers, d_model 4096, V 126 464; stage-1 call of
1 x 512 tokens and verification call of 4 x 512), config 4 (28 layers, grouped KV heads with QKV bias,
V 152 064; 1 x 1024 and 6 x 1024) and config 5 (config 3's model; 16 x 1280 and 128 x 1280 tokens, block 64).

The oracle needs 12-35 s per sequence-forward on 16 host cores and the fp32 host copy of the weights about
32 GB, so each batch is compared on sampled sequences only (every sequence runs through the same kernels), and
the same sequence sits in both the stage-1-shaped and the verification-shaped batch, so that one oracle
evaluation checks both launch configurations.  At these widths the logit tolerance is calibrated by the oracle
itself (check_sequence in test_gpu_forward.py): no bf16 evaluation of these networks stays within 2e-2 of exact
arithmetic."""
import time

import numpy as np
import pytest

import psd_inputs as inp
from oracle import psd_oracle as orc

pytestmark = pytest.mark.gpu


def _state(shape, N, block_start, L, seed, n_committed):
    rng = np.random.default_rng(seed)
    t = np.full(N, shape.mask_id, dtype=np.int32)
    t[:block_start] = inp.draw_prompt(shape.vocab, block_start, seed)
    idx = rng.choice(L, size=n_committed, replace=False)
    t[block_start + idx] = rng.integers(0, shape.vocab - 1, size=n_committed)
    return t


def _need_memory():
    import psutil
    if psutil.virtual_memory().available < 60 * 2 ** 30:
        pytest.skip("needs about 40 GB of free host memory for the fp32 host copy of a 7-8B-parameter model")


def test_config3_full_depth_stage1_and_verify():
    _need_memory()
    import paper_2605_15609_amd as psd
    from tests.gpu_common import say
    from tests.test_gpu_forward import _compare
    w = inp.WORKLOADS[3]
    shape, N, P, L, K = w.shape, w.seq_len, w.prompt_len, w.block_len, w.n_drafts
    t0 = time.perf_counter()
    host = inp.draw_model(shape, N, threads=16)
    model = psd.Model.from_host(host)
    say(f"[full-size] config 3 drawn and uploaded after {time.perf_counter() - t0:.0f} s")
    tokens = inp.initial_state(w)[0]
    _compare(model, host, [tokens], P, L, 2e-2, "cfg3-full/stage-1", calibrate=True)
    say(f"[full-size] stage-1 compared after {time.perf_counter() - t0:.0f} s")
    # drafts from the oracle's own stage-1 decisions (Eq. 1, Eq. 2), then the batched verification call
    top1, conf = orc.forward_confidence(host, tokens, P, L)
    policy, graph = orc.Policy(w.tau, w.k_min, w.k_max), orc.chain_graph(K)
    committed, _ = orc.select_unmask(tokens, P, L, top1, conf, policy, shape.mask_id)
    sigma, m, drafts = orc.build_drafts(committed, P, L, top1, conf, graph, shape.mask_id)
    assert m >= K - 1, "the first block leaves enough masks for every draft to differ"
    say(f"[full-size] drafts built after {time.perf_counter() - t0:.0f} s")
    _compare(model, host, [np.asarray(d, dtype=np.int32) for d in drafts], P, L, 2e-2, "cfg3-full/verify", check=(0, K - 1),
             calibrate=True)
    say(f"[full-size] verification compared after {time.perf_counter() - t0:.0f} s")
    model.close()


@pytest.mark.parametrize("cfg", [4, 5])
def test_full_depth_both_launch_shapes_on_a_shared_sequence(cfg):
    _need_memory()
    import paper_2605_15609_amd as psd
    from tests.gpu_common import say
    from tests.test_gpu_forward import check_sequence, hip_forward, oracle_reference
    w = inp.WORKLOADS[cfg]
    shape, N, L, K, B = w.shape, w.seq_len, w.block_len, w.n_drafts, w.batch
    bs = w.prompt_len + L            # second block: one finished block precedes it
    t0 = time.perf_counter()
    host = inp.draw_model(shape, N, threads=16)
    model = psd.Model.from_host(host)
    say(f"[full-size] config {cfg} drawn and uploaded after {time.perf_counter() - t0:.0f} s")
    # seeded states with the block partly committed; sequence 0 of both batches is the same
    states = [_state(shape, N, bs, L, 100 + i, (7 * i + 5) % L) for i in range(B * K)]
    for t in states:
        t[w.prompt_len: bs] = inp.draw_prompt(shape.vocab, L, 999)     # the finished first block
    ref = oracle_reference(host, states[0], bs, L, calibrate=True)
    say(f"[full-size] oracle evaluated sequence 0 after {time.perf_counter() - t0:.0f} s")
    for label, batch in ((f"cfg{cfg}-full/stage-1 shape ({B} x {N})", states[:B]),
                         (f"cfg{cfg}-full/verify shape ({B * K} x {N})", states)):
        logits, top1, conf = hip_forward(model, batch, bs, L)
        err, tol, near, wide = check_sequence(ref, logits[0], top1[0], conf[0], states[0], shape.mask_id, bs, L, 2e-2, label)
        say(f"[full-size] {label}: logits max-abs err {err:.3e} (tol {tol:.3e}), near-ties {near}, inside the band {wide}; "
            f"{time.perf_counter() - t0:.0f} s")
        del logits
    model.close()


def test_config3_full_depth_block_causal_with_kv_cache():
    """The same 8B-parameter shape as a context-causal block model: prefill of the prompt and one finished block
    into the KV cache, then the block-row model call in both launch shapes (1 x 32 rows; 4 drafts x 32 rows sharing
    the cache) against the oracle's masked whole-sequence forward."""
    _need_memory()
    import dataclasses
    import torch
    import paper_2605_15609_amd as psd
    from tests.gpu_common import say, to_dev
    from tests.test_gpu_forward import check_sequence
    w = inp.WORKLOADS[3]
    shape = dataclasses.replace(w.shape, attention="block_causal")
    N, L, K = w.seq_len, w.block_len, w.n_drafts
    start = w.prompt_len + L
    t0 = time.perf_counter()
    host = inp.draw_model(shape, N, threads=16)
    model = psd.Model.from_host(host)
    say(f"[full-size] block-causal config 3 drawn and uploaded after {time.perf_counter() - t0:.0f} s")
    states = [_state(shape, N, start, L, 300 + i, 3 + 5 * i) for i in range(K)]
    for t in states:
        t[:start] = states[0][:start]                     # the drafts of one sequence share everything before the block
    cache = psd.KvCache(model, 1, N)
    psd.psd_kv_prefill(model, to_dev(states[0][None]), start, L, cache)
    o_top1, o_conf, z = orc.forward_confidence(host, states[0], start, L, return_logits=True, block_causal=True)
    z_b = orc.block_logits(host, states[0], start, L, operands="bf16", block_causal=True)
    say(f"[full-size] oracle evaluated draft 0 after {time.perf_counter() - t0:.0f} s")
    for label, batch in (("cfg3-block-causal/stage-1 shape (1 x 32 rows)", states[:1]),
                         (f"cfg3-block-causal/verify shape ({K} x 32 rows, shared cache)", states)):
        top1, conf, logits = psd.psd_forward_confidence_cached(model, to_dev(np.stack(batch)), start, L, cache,
                                                               seqs_per_cache=len(batch), want_logits=True)
        torch.cuda.synchronize()
        logits = logits.cpu().numpy().reshape(len(batch), L, -1)
        err, tol, near, wide = check_sequence((o_top1, o_conf, z, z_b), logits[0], top1[0].cpu().numpy(), conf[0].cpu().numpy(),
                                              states[0], shape.mask_id, start, L, 2e-2, label)
        say(f"[full-size] {label}: logits max-abs err {err:.3e} (tol {tol:.3e}), near-ties {near}, inside the band {wide}; "
            f"{time.perf_counter() - t0:.0f} s")
    model.close()


def test_config3_full_depth_approximate_cache():
    """Config 3 itself (bidirectional) under the approximate prefix + suffix cache: the exact call that enters a block
    fills the cache; then the block-row call in both launch shapes (1 x 32 rows; 4 drafts x 32 rows sharing the cache)
    after five commits, against the oracle's ApproximateCache in exact arithmetic, with the tolerance calibrated by
    the same oracle mode on bf16 operands."""
    _need_memory()
    import torch
    import paper_2605_15609_amd as psd
    from tests.gpu_common import say, to_dev
    from tests.test_gpu_forward import check_sequence
    w = inp.WORKLOADS[3]
    shape = w.shape
    N, L, K = w.seq_len, w.block_len, w.n_drafts
    start = w.prompt_len + L
    t0 = time.perf_counter()
    host = inp.draw_model(shape, N, threads=16)
    model = psd.Model.from_host(host)
    say(f"[full-size] config 3 drawn and uploaded after {time.perf_counter() - t0:.0f} s")
    entry = np.full(N, shape.mask_id, dtype=np.int32)
    entry[:start] = inp.draw_prompt(shape.vocab, start, 300)
    exact, rounded = orc.ApproximateCache(host), orc.ApproximateCache(host, operands="bf16")
    ref0 = exact(entry, start, L)
    z0 = exact.logits.copy()
    rounded(entry, start, L)
    zb0 = rounded.logits.copy()
    say(f"[full-size] oracle refresh calls done after {time.perf_counter() - t0:.0f} s")
    cache = psd.KvCache(model, 1, N - L)
    top1, conf, logits = psd.psd_forward_confidence_approx(model, to_dev(entry[None]), start, L, cache, refresh=True,
                                                           want_logits=True)
    torch.cuda.synchronize()
    err, tol, near, wide = check_sequence((ref0[0], ref0[1], z0, zb0), logits.cpu().numpy(), top1[0].cpu().numpy(),
                                          conf[0].cpu().numpy(), entry, shape.mask_id, start, L, 2e-2, "cfg3-approx/refresh")
    say(f"[full-size] cfg3-approx/refresh: logits max-abs err {err:.3e} (tol {tol:.3e}), near-ties {near}, inside the band {wide}")
    rng = np.random.default_rng(5)
    t1 = entry.copy()
    idx = rng.choice(L, size=5, replace=False)
    t1[start + idx] = ref0[0][idx]
    drafts = np.repeat(t1[None], K, axis=0)
    order = [j for j in range(L) if t1[start + j] == shape.mask_id]
    for k in range(1, K):
        for j in order[:k]:
            drafts[k, start + j] = ref0[0][j]
    ref1 = exact(drafts[K - 1], start, L)          # the deepest draft: it differs most from the state the cache was filled on
    z1 = exact.logits.copy()
    rounded(drafts[K - 1], start, L)
    zb1 = rounded.logits.copy()
    for label, batch, row in ((f"cfg3-approx/stage-1 shape (1 x {L} rows)", drafts[K - 1:], 0),
                              (f"cfg3-approx/verify shape ({K} x {L} rows, shared cache)", drafts, K - 1)):
        top1, conf, logits = psd.psd_forward_confidence_approx(model, to_dev(batch), start, L, cache, refresh=False,
                                                               seqs_per_cache=len(batch), want_logits=True)
        torch.cuda.synchronize()
        logits = logits.cpu().numpy().reshape(len(batch), L, -1)
        err, tol, near, wide = check_sequence((ref1[0], ref1[1], z1, zb1), logits[row], top1[row].cpu().numpy(),
                                              conf[row].cpu().numpy(), drafts[K - 1], shape.mask_id, start, L, 2e-2, label)
        say(f"[full-size] {label}: logits max-abs err {err:.3e} (tol {tol:.3e}), near-ties {near}, inside the band {wide}; "
            f"{time.perf_counter() - t0:.0f} s")
    model.close()
