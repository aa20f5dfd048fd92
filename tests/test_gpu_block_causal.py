"""Context-causal block attention (one model family of the paper, App. A) with an exact prefix KV cache.

The oracle defines the mode as one masked forward over the whole sequence; the HIP product path runs the block
rows alone against cached keys and values.  Checked here: (1) the masked whole-sequence forward on the plain
kernels, (2) prefill + cached forward (stage-1 shape and a verification batch whose drafts share one cache)
against the oracle's masked forward, fp32 within 1e-4 and bf16 within 2e-2, (3) the cached path equals the
masked whole-sequence path on the device, (4) a free-running fp32 decode with the cache reproduces the oracle's
decode token for token, (5) a batched cached decode equals the sequences decoded alone."""
import dataclasses

import numpy as np
import pytest
import torch

import psd_inputs as inp
from oracle import psd_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _bc(shape, **kw):
    return dataclasses.replace(shape, attention="block_causal", **kw)


FP32 = _bc(inp.cut_down(inp.WORKLOADS[4].shape, name="bc-fp32", dtype="fp32", n_layers=2, d_model=96, n_heads=6, n_kv_heads=2,
                        d_head=16, d_ffn=160, vocab=211, seed=41))
BF16 = {
    "mha-dh64": _bc(inp.cut_down(inp.WORKLOADS[2].shape, n_layers=2, vocab=5000, seed=42)),
    "gqa-bias-dh128": _bc(inp.cut_down(inp.WORKLOADS[4].shape, n_layers=2, d_model=512, n_heads=4, n_kv_heads=2, d_ffn=640,
                                       vocab=3001, seed=43)),
}


def _state(shape, N, P, L, block, seed, n_committed):
    """prompt, `block` finished generation blocks, an active block with n_committed tokens, masks behind."""
    rng = np.random.default_rng(seed)
    t = np.full(N, shape.mask_id, dtype=np.int32)
    start = P + block * L
    t[:start] = inp.draw_prompt(shape.vocab, start, seed)
    idx = rng.choice(L, size=n_committed, replace=False)
    t[start + idx] = rng.integers(0, shape.vocab - 1, size=n_committed)
    return t, start


def _check(shape, host, logits, top1, conf, t, start, L, tol, label):
    from tests.test_gpu_forward import check_sequence
    o_top1, o_conf, z = orc.forward_confidence(host, t, start, L, return_logits=True, block_causal=True)
    return check_sequence((o_top1, o_conf, z, None), logits, top1, conf, t, shape.mask_id, start, L, tol, label)


@pytest.mark.parametrize("L", [16, 32, 64])
def test_fp32_cached_and_masked_paths_match_the_oracle(L):
    import paper_2605_15609_amd as psd
    from tests.gpu_common import say
    shape = FP32
    P, N = 2 * L, 5 * L
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    cache = psd.KvCache(model, 1, N)
    for block in (0, 2):
        t, start = _state(shape, N, P, L, block, 7 + block, L // 3)
        d = _dev(t[None])
        # masked attention over the whole sequence (plain kernels)
        logits = psd.psd_forward_logits(model, d, start, L).cpu().numpy()
        top1, conf = psd.psd_forward_confidence(model, d, start, L)
        e1 = _check(shape, host, logits, top1[0].cpu().numpy(), conf[0].cpu().numpy(), t, start, L, 1e-4, f"fp32 masked L={L}")[0]
        # the block rows against the prefix cache
        cache.reset()
        psd.psd_kv_prefill(model, d, start, L, cache)
        c_top1, c_conf, c_logits = psd.psd_forward_confidence_cached(model, d, start, L, cache, want_logits=True)
        e2 = _check(shape, host, c_logits.cpu().numpy(), c_top1[0].cpu().numpy(), c_conf[0].cpu().numpy(), t, start, L, 1e-4,
                    f"fp32 cached L={L}")[0]
        say(f"[block-causal] fp32 L={L} block {block}: logits max-abs err masked {e1:.2e}, cached {e2:.2e}")


@pytest.mark.parametrize("name", list(BF16))
@pytest.mark.parametrize("plain", [0, 7], ids=["mfma", "plain"])
def test_bf16_cached_forward_matches_the_oracle_and_the_masked_device_path(name, plain):
    import paper_2605_15609_amd as psd
    from tests.gpu_common import say
    shape = BF16[name]
    L, K = 32, 4
    P, N = 3 * L, 6 * L
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    model.set_plain(plain)
    cache = psd.KvCache(model, 2, N)
    # two sequences with their own prompts and one finished generation block each
    seqs = [_state(shape, N, P, L, 1, 20 + b, 5 + 3 * b) for b in range(2)]
    start = seqs[0][1]
    d = _dev(np.stack([t for t, _ in seqs]))
    psd.psd_kv_prefill(model, d, start, L, cache)
    top1, conf, logits = psd.psd_forward_confidence_cached(model, d, start, L, cache, want_logits=True)
    logits = logits.cpu().numpy().reshape(2, L, -1)
    for b, (t, _) in enumerate(seqs):
        err = _check(shape, host, logits[b], top1[b].cpu().numpy(), conf[b].cpu().numpy(), t, start, L, 2e-2,
                     f"{name} cached stage-1 seq {b}")[0]
        say(f"[block-causal] {name} plain={plain} stage-1 seq {b}: logits max-abs err {err:.3e}")
    # a verification batch: K drafts per sequence sharing that sequence's cache
    rng = np.random.default_rng(5)
    drafts = []
    for b, (t, _) in enumerate(seqs):
        for k in range(K):
            dft = t.copy()
            masked = np.nonzero(dft[start: start + L] == shape.mask_id)[0]
            fill = masked[: 2 * k]
            dft[start + fill] = rng.integers(0, shape.vocab - 1, size=len(fill))
            drafts.append(dft)
    dd = _dev(np.stack(drafts))
    v_top1, v_conf, v_logits = psd.psd_forward_confidence_cached(model, dd, start, L, cache, seqs_per_cache=K, want_logits=True)
    v_logits = v_logits.cpu().numpy().reshape(2 * K, L, -1)
    for i in (1, K - 1, K + 2, 2 * K - 1):
        err = _check(shape, host, v_logits[i], v_top1[i].cpu().numpy(), v_conf[i].cpu().numpy(), drafts[i], start, L, 2e-2,
                     f"{name} cached verify draft {i}")[0]
        say(f"[block-causal] {name} plain={plain} verify draft {i}: logits max-abs err {err:.3e}")
    # the masked whole-sequence forward on the device agrees with the cached one to rounding
    m_logits = psd.psd_forward_logits(model, dd, start, L).cpu().numpy().reshape(2 * K, L, -1)
    assert np.abs(m_logits - v_logits).max() < 2e-2


@pytest.mark.parametrize("name", list(BF16))
def test_bf16_cached_forward_does_not_depend_on_what_the_cache_memory_held(name):
    """Only the first block_start slots of a cache are context.  With the rest of the cache memory holding NaN bit patterns
    (an allocation nobody cleared) the result must be bit-identical to the one over a cleared cache: the last, partial key
    tile of the prefix reads value slots past the end, and 0 x NaN would poison every query."""
    import paper_2605_15609_amd as psd
    shape = BF16[name]
    L = 32
    P, N = 3 * L, 6 * L                                    # a prefix of 96 keys: one full 64-key tile and a half
    model = psd.Model.from_host(inp.draw_model(shape, N), DEV)
    t, start = _state(shape, N, P, L, 0, 33, 6)
    d = _dev(np.stack([t, t]))
    results = []
    for poison in (False, True):
        cache = psd.KvCache(model, 2, N)
        if poison:
            cache.mem.fill_(0xff)                          # bf16 0xffff: a NaN in every slot
        psd.psd_kv_prefill(model, d, start, L, cache)
        top1, conf, logits = psd.psd_forward_confidence_cached(model, d, start, L, cache, want_logits=True)
        results.append((top1.cpu().numpy(), conf.cpu().numpy(), logits.cpu().numpy()))
    assert np.isfinite(results[1][2]).all()
    for a, b in zip(results[0], results[1]):
        assert (a == b).all()


def test_fp32_free_running_cached_decode_matches_the_oracle_decode():
    import paper_2605_15609_amd as psd
    shape = FP32
    L, P, G = 16, 32, 48
    N = P + G
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    for K, tau in ((3, 0.9), (4, 0.05), (1, 0.9)):
        tokens0 = np.full((1, N), shape.mask_id, dtype=np.int32)
        tokens0[0, :P] = inp.draw_prompt(shape.vocab, P, 61)
        d = _dev(tokens0)
        cache = psd.KvCache(model, 1, N)
        psd.psd_kv_prefill(model, d, P, L, cache)
        stats = [psd.Stats()]
        for start in range(P, N, L):
            stats = psd.psd_decode_block_cached(model, d, start, L, psd.Policy(tau, 1, 0), psd.chain_graph(K), cache, stats)
        ref, ostats = orc.decode(orc.model_confidence_fn(host, block_causal=True), tokens0[0], P, L, orc.Policy(tau, 1, 0),
                                 orc.chain_graph(K), shape.mask_id)
        assert (d.cpu().numpy()[0] == ref).all(), (K, tau)
        s = stats[0]
        assert (s.invocations, s.tokens_policy, s.tokens_draft, s.tokens_postverify) == \
               (ostats.invocations, ostats.tokens_policy, ostats.tokens_draft, ostats.tokens_postverify)
        assert s.depth_hist[:32] == ostats.depth_hist
        # EOS early stopping (App. B.1) on the cached path: an EOS id the free run produces in its second block
        eos = int(ref[P + L + 5])
        d = _dev(tokens0)
        cache.reset()
        psd.psd_kv_prefill(model, d, P, L, cache)
        stats = [psd.Stats()]
        for start in range(P, N, L):
            if stats[0].stopped:
                break
            stats = psd.psd_decode_block_cached(model, d, start, L, psd.Policy(tau, 1, 0, eos_id=eos), psd.chain_graph(K), cache,
                                                stats)
        ref2, o2 = orc.decode(orc.model_confidence_fn(host, block_causal=True), tokens0[0], P, L, orc.Policy(tau, 1, 0),
                              orc.chain_graph(K), shape.mask_id, eos_id=eos)
        s = stats[0]
        assert (d.cpu().numpy()[0] == ref2).all() and o2.stopped, (K, tau)
        assert (s.invocations, s.tokens, s.tokens_counted, bool(s.stopped), s.eos_pos) == \
               (o2.invocations, o2.tokens, o2.tokens_counted, o2.stopped, o2.eos_pos)


def test_fp32_single_forward_cached_decode_matches_the_oracle_variant():
    """The single-forward loop on the KV-cached model calls: tokens and counters equal the oracle's single-forward decode
    with the block-causal model, block by block."""
    import paper_2605_15609_amd as psd
    shape = FP32
    L, P, G = 16, 32, 48
    N = P + G
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    for K, tau in ((3, 0.9), (4, 0.05)):
        tokens0 = np.full((1, N), shape.mask_id, dtype=np.int32)
        tokens0[0, :P] = inp.draw_prompt(shape.vocab, P, 61)
        d = _dev(tokens0)
        cache = psd.KvCache(model, 1, N)
        psd.psd_kv_prefill(model, d, P, L, cache)
        stats = [psd.Stats()]
        for start in range(P, N, L):
            stats = psd.psd_decode_block_cached(model, d, start, L, psd.Policy(tau, 1, 0, single_forward=True), psd.chain_graph(K),
                                                cache, stats)
        ref, ostats = orc.decode(orc.model_confidence_fn(host, block_causal=True), tokens0[0], P, L, orc.Policy(tau, 1, 0),
                                 orc.chain_graph(K), shape.mask_id, single_forward=True)
        assert (d.cpu().numpy()[0] == ref).all(), (K, tau)
        s = stats[0]
        assert (s.invocations, s.tokens_policy, s.tokens_draft, s.tokens_postverify) == \
               (ostats.invocations, ostats.tokens_policy, ostats.tokens_draft, ostats.tokens_postverify)
        assert s.invocations == G // L + sum(s.depth_hist)


def test_bf16_batched_cached_decode_equals_sequences_alone_and_the_masked_decode():
    import paper_2605_15609_amd as psd
    shape = dataclasses.replace(BF16["mha-dh64"], logit_scale=14.0)
    L, P, G, K, B = 32, 64, 64, 2, 2     # every model call of both runs stays within 128 rows (same K-split, same sums)
    N = P + G
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    policy, graph = psd.Policy(0.9, 1, 0), psd.chain_graph(K)
    tokens = np.full((B, N), shape.mask_id, dtype=np.int32)
    for b in range(B):
        tokens[b, :P] = inp.draw_prompt(shape.vocab, P, 70 + b)

    def run(batch):
        d = _dev(batch)
        cache = psd.KvCache(model, batch.shape[0], N)
        psd.psd_kv_prefill(model, d, P, L, cache)
        stats = [psd.Stats() for _ in range(batch.shape[0])]
        for start in range(P, N, L):
            stats = psd.psd_decode_block_cached(model, d, start, L, policy, graph, cache, stats)
        return d.cpu().numpy(), stats

    together, st_all = run(tokens)
    assert not (together == shape.mask_id).any()
    for b in range(B):
        alone, st = run(tokens[b: b + 1])
        assert (alone[0] == together[b]).all()
        assert st[0].invocations == st_all[b].invocations and st[0].tokens == st_all[b].tokens == G


def test_bf16_cached_call_at_128_and_256_rows_agrees_to_rounding():
    """Block-row calls over at most 128 rows cut the residual contractions along K (a weight stream needs the workgroups),
    larger ones do not: a sequence's fp32 sums, hence its logits, depend on whether 4 or 8 sequences share the call --
    to rounding, not beyond.  Both stay within the logit tolerance of each other and of the oracle; exact batch
    invariance is a property of the whole-sequence calls only."""
    import paper_2605_15609_amd as psd
    from tests.gpu_common import say
    shape = BF16["gqa-bias-dh128"]
    L = 32
    P, N = 2 * L, 4 * L
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    seqs = [_state(shape, N, P, L, 0, 50 + b, 3 + b) for b in range(8)]
    start = seqs[0][1]
    tokens = np.stack([t for t, _ in seqs])
    out = {}
    for S in (4, 8):
        d = _dev(tokens[:S])
        cache = psd.KvCache(model, S, N)
        psd.psd_kv_prefill(model, d, start, L, cache)
        top1, conf, logits = psd.psd_forward_confidence_cached(model, d, start, L, cache, want_logits=True)
        out[S] = (top1.cpu().numpy(), conf.cpu().numpy(), logits.cpu().numpy().reshape(S, L, -1))
    diff = float(np.abs(out[4][2] - out[8][2][:4]).max())
    say(f"[block-causal] 128-row call (K-split) vs 256-row call: logits differ by {diff:.3e}; bit-identical: {diff == 0.0}")
    assert diff <= 2e-2
    for S in (4, 8):
        _check(shape, host, out[S][2][1], out[S][0][1], out[S][1][1], seqs[1][0], start, L, 2e-2, f"cached call of {S} sequences")
    masked = tokens[:4, start: start + L] == shape.mask_id
    rel = np.abs(out[4][1][masked] / out[8][1][:4][masked] - 1.0).max()
    assert rel <= np.expm1(2 * 2e-2)


def test_empty_prefix_full_cache_and_argument_errors():
    import paper_2605_15609_amd as psd
    shape = FP32
    L = 16
    N = 3 * L
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    cache = psd.KvCache(model, 1, N)
    # no prompt at all: the first block sees only itself
    t = np.full(N, shape.mask_id, dtype=np.int32)
    t[3] = 5
    d = _dev(t[None])
    psd.psd_kv_prefill(model, d, 0, L, cache)
    top1, conf, logits = psd.psd_forward_confidence_cached(model, d, 0, L, cache, want_logits=True)
    _check(shape, host, logits.cpu().numpy(), top1[0].cpu().numpy(), conf[0].cpu().numpy(), t, 0, L, 1e-4, "empty prefix")
    # the last block of a cache filled to capacity
    t2, start = _state(shape, N, 2 * L, L, 0, 9, 4)
    d2 = _dev(t2[None])
    cache.reset()
    psd.psd_kv_prefill(model, d2, start, L, cache)
    top1, conf, logits = psd.psd_forward_confidence_cached(model, d2, start, L, cache, want_logits=True)
    _check(shape, host, logits.cpu().numpy(), top1[0].cpu().numpy(), conf[0].cpu().numpy(), t2, start, L, 1e-4, "cache at capacity")
    # errors are reported, nothing is launched
    with pytest.raises(psd.PsdError):
        psd.psd_forward_confidence_cached(model, d2, start + 4, L, cache)            # block not aligned
    with pytest.raises(psd.PsdError):
        psd.psd_kv_prefill(model, d2, L + 3, L, cache)                               # prompt not a multiple of L
    with pytest.raises(psd.PsdError):
        psd.psd_forward_confidence_cached(model, d2, start, 8, cache)                # block length not a multiple of 16
    small = psd.KvCache(model, 1, 2 * L)
    with pytest.raises(psd.PsdError):
        psd.psd_forward_confidence_cached(model, d2, start, L, small)                # block beyond the cache capacity
    bidir = psd.Model.from_host(inp.draw_model(dataclasses.replace(shape, attention="bidirectional"), N), DEV)
    with pytest.raises(psd.PsdError):
        psd.psd_forward_confidence_cached(bidir, d2, start, L, psd.KvCache(bidir, 1, N))   # exact only for block-causal models


def test_graph_calibration_on_the_cached_path_scores_like_the_oracle():
    import paper_2605_15609_amd as psd
    shape = FP32
    L, P, G, B = 16, 32, 32, 2
    N = P + G
    host = inp.draw_model(shape, N)
    model = psd.Model.from_host(host, DEV)
    tokens0 = np.full((B, N), shape.mask_id, dtype=np.int32)
    for b in range(B):
        tokens0[b, :P] = inp.draw_prompt(shape.vocab, P, 90 + b)
    cands = [psd.chain_graph(1), psd.chain_graph(3), psd.lattice_graph(2)]
    d = _dev(tokens0)
    cache = psd.KvCache(model, B, N)
    best, scores = psd.psd_calibrate_graph(model, d, P, L, psd.Policy(0.05, 1, 0), cands, cache)
    assert (d.cpu().numpy() == tokens0).all()
    fn = orc.model_confidence_fn(host, block_causal=True)
    for g, sc in zip(cands, scores):
        og = orc.Graph(tuple(frozenset(r for r in range(64) if (rs >> r) & 1) for rs in g.rank_sets))
        tok = inv = 0
        for b in range(B):
            _, st = orc.decode(fn, tokens0[b], P, L, orc.Policy(0.05, 1, 0), og, shape.mask_id)
            tok, inv = tok + st.tokens, inv + st.invocations
        assert (sc["tokens"], sc["invocations"]) == (tok, inv) and sc["seconds"] > 0
    assert best == max(range(len(cands)), key=lambda c: (scores[c]["tokens_per_s"], -c))
