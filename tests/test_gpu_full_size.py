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


# ------------------------------------------------------------------------------------------------------------
# One layer at a time, stage by stage, at full width: the check that an end-to-end tolerance of 0.2 logits cannot give.
# The HIP layer runs alone (psd_debug_layer) on the ORACLE's exact residual stream at the input of an early, a middle
# and the last layer of the 32-layer model; every stage's output is then compared with the exact (fp64) evaluation
# of that stage on the HIP path's own input of the stage.  So each comparison sees exactly one bf16 rounding of the
# stage's result (unit round-off u = 2^-8, relative) plus fp32 accumulation, and the bounds below are those:
#   a    = bf16(rmsnorm(h))                         |err| <= u |ref|
#   q, k = bf16(rope(bf16(a Wq^T)))                 |err| <= u (|x1 c| + |x2 s|) + u |ref|     (the projection is stored in
#                                                    bf16 before the rotation: two roundings)
#   v    = bf16(a Wv^T)                             |err| <= u |ref|
#   o    = bf16(sum_j bf16(p_j) v_j / sum_j p_j)    |err| <= u sum_j p_j |v_j| / sum_j p_j + u |ref|
#   a2   = bf16(rmsnorm(h + o Wo^T))                |err| <= u |ref|
#   act  = bf16(silu(a2 Wg^T) * (a2 Wu^T))          |err| <= u |ref|
#   h'   = h + o Wo^T + act Wd^T  (fp32)            |err| <= fp32 accumulation only
# each plus the fp32 accumulation term g(K) sum_k |x_k w_k| with g(K) = 4 sqrt(K) 2^-24.
LAYERS_CHECKED = (0, 15, 31)
U = 2.0 ** -8


def _acc(K):
    return 4.0 * np.sqrt(K) * 2.0 ** -24


def _stage_check(name, got, ref, bound, stats):
    err = np.abs(got - ref)
    worst = float((err / np.maximum(bound, 1e-300)).max())
    stats[name] = round(worst, 3)
    assert (err <= bound).all(), f"{name}: error {err.max():.3e} exceeds its bound by a factor {worst:.2f} at {np.unravel_index((err / np.maximum(bound, 1e-300)).argmax(), err.shape)}"


def test_config3_single_layers_stage_by_stage_against_unit_roundoff_bounds():
    _need_memory()
    import torch
    import paper_2605_15609_amd as psd
    from paper_2605_15609_amd import binding as B
    from tests.gpu_common import say, to_dev
    w = inp.WORKLOADS[3]
    shape, N, P, L = w.shape, w.seq_len, w.prompt_len, w.block_len
    H, Hkv, dh, d, F = shape.n_heads, shape.n_kv_heads, shape.d_head, shape.d_model, shape.d_ffn
    t0 = time.perf_counter()
    host = inp.draw_model(shape, N, threads=16)
    model = psd.Model.from_host(host)
    say(f"[layer] config 3 drawn and uploaded after {time.perf_counter() - t0:.0f} s")
    tokens = _state(shape, N, P, L, 77, 9)
    cos, sin = host.rope_cos[:N].astype(np.float64), host.rope_sin[:N].astype(np.float64)
    h = host.tok_emb[tokens].astype(np.float64)
    inputs = {}
    for l, lw in enumerate(host.layers):
        if l in LAYERS_CHECKED:
            inputs[l] = h.astype(np.float32)        # the stream crosses the boundary as fp32
        if l == max(LAYERS_CHECKED):
            break
        h = orc.layer_forward(h, lw, shape, cos, sin)
    say(f"[layer] oracle residual streams at the inputs of layers {LAYERS_CHECKED} after {time.perf_counter() - t0:.0f} s")
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    for l in LAYERS_CHECKED:
        lw = host.layers[l]
        W = lambda k: lw[k].astype(np.float64)
        h_in = inputs[l].astype(np.float64)
        stats = {}
        # ---- first half: norm, projections, rotary, attention
        d_h = to_dev(inputs[l])
        out = B.debug_layer(model, l, d_h, 1, N, L, stop_after=1)
        torch.cuda.synchronize()
        assert torch.equal(d_h.cpu(), torch.from_numpy(inputs[l])), "stop_after = 1 must leave the stream untouched"
        a1, qkv, o = f64(out["a"]), f64(out["qkv"]), f64(out["o"])
        ref = orc.rmsnorm(h_in, W("attn_norm"), shape.rms_eps)
        _stage_check("a", a1, ref, U * np.abs(ref) * 1.001 + 1e-12, stats)
        Wqkv = np.concatenate([W("wq"), W("wk"), W("wv")])
        pre = a1 @ Wqkv.T
        accb = _acc(d) * (np.abs(a1) @ np.abs(Wqkv).T)
        nq, nk = H * dh, Hkv * dh
        qk_room = np.zeros((N, nq + nk))          # |x1 c| + |x2 s| + |result| of every rotated element
        qk_acc = np.zeros((N, nq + nk))           # fp32 accumulation room of every rotated element
        for name, lo, nh in (("q", 0, H), ("k", nq, Hkv)):
            x = pre[:, lo: lo + nh * dh].reshape(N, nh, dh)
            ab = accb[:, lo: lo + nh * dh].reshape(N, nh, dh)
            half = dh // 2
            x1, x2, c, s_ = x[..., :half], x[..., half:], cos[:, None, :], sin[:, None, :]
            ref = orc.rope(x, cos, sin)
            spread = np.concatenate([np.abs(x1 * c) + np.abs(x2 * s_), np.abs(x2 * c) + np.abs(x1 * s_)], axis=-1)
            acc_r = np.concatenate([ab[..., :half] + ab[..., half:]] * 2, axis=-1)
            _stage_check(name, qkv[:, lo: lo + nh * dh].reshape(N, nh, dh), ref, U * (spread + np.abs(ref)) * 1.001 + acc_r + 1e-12, stats)
            qk_room[:, lo: lo + nh * dh] = (spread + np.abs(ref)).reshape(N, nh * dh)
            qk_acc[:, lo: lo + nh * dh] = acc_r.reshape(N, nh * dh)
        ref = pre[:, nq + nk:]
        _stage_check("v", qkv[:, nq + nk:], ref, U * np.abs(ref) * 1.001 + accb[:, nq + nk:] + 1e-12, stats)
        q, k, v = qkv[:, :nq].reshape(N, H, dh), qkv[:, nq: nq + nk].reshape(N, Hkv, dh), qkv[:, nq + nk:].reshape(N, Hkv, dh)
        ref = orc.attention(q, k, v).reshape(N, H * dh)
        spread = orc.attention(q, k, np.abs(v)).reshape(N, H * dh)        # sum_j p_j |v_j| / sum_j p_j
        _stage_check("o", o, ref, U * (spread + np.abs(ref)) * 1.001 + 1e-4 * spread + 1e-12, stats)
        # ---- whole layer: same first half (deterministic), then output projection, norm, SwiGLU, down projection
        d_h = to_dev(inputs[l])
        out = B.debug_layer(model, l, d_h, 1, N, L, stop_after=0)
        torch.cuda.synchronize()
        assert torch.equal(out["o"].cpu(), torch.from_numpy(o.astype(np.float32)).to(torch.bfloat16)), "the first half is not repeatable"
        a2, act, h_out = f64(out["a"]), f64(out["act"]), d_h.cpu().numpy().astype(np.float64)
        upd_o = o @ W("wo").T
        h_mid = h_in + upd_o
        acc_o = _acc(H * dh) * (np.abs(o) @ np.abs(W("wo")).T) + 2.0 ** -23 * np.abs(h_mid)
        ref = orc.rmsnorm(h_mid, W("ffn_norm"), shape.rms_eps)
        rms = np.sqrt(np.mean(h_mid ** 2, axis=-1, keepdims=True))
        _stage_check("a2", a2, ref, U * np.abs(ref) * 1.001 + 2.0 * acc_o / rms + 1e-12, stats)
        g, u_ = a2 @ W("w_gate").T, a2 @ W("w_up").T
        ref = orc.silu(g) * u_
        ag, au = _acc(d) * (np.abs(a2) @ np.abs(W("w_gate")).T), _acc(d) * (np.abs(a2) @ np.abs(W("w_up")).T)
        _stage_check("act", act, ref, U * np.abs(ref) * 1.001 + 1.2 * ag * np.abs(u_) + au * np.abs(orc.silu(g)) + 1e-12, stats)
        ref = h_mid + act @ W("w_down").T
        acc_d = _acc(F) * (np.abs(act) @ np.abs(W("w_down")).T)
        _stage_check("h_out", h_out, ref, acc_o + acc_d + 2.0 ** -22 * np.abs(ref) + 1e-12, stats)
        # ---- the same layer on the plain fp32-accumulating debug kernels: the two paths round at the same points, so
        # they may differ by the last bit of a bf16 result here and there, nothing more
        model.set_plain(7)
        d_p = to_dev(inputs[l])
        outp = B.debug_layer(model, l, d_p, 1, N, L, stop_after=0)
        torch.cuda.synchronize()
        model.set_plain(0)
        qkv_p, o_p, act_p = f64(outp["qkv"]), f64(outp["o"]), f64(outp["act"])
        ulp = lambda x, y: 2.0 ** -7 * np.maximum(np.abs(x), np.abs(y))
        # (a result that cancels to almost nothing is smaller than the accumulation error of its sum: both paths get that room)
        pairs = (("v", qkv[:, nq + nk:], qkv_p[:, nq + nk:], 1.01 * ulp(qkv[:, nq + nk:], qkv_p[:, nq + nk:]) + 2 * accb[:, nq + nk:]),
                 ("qk", qkv[:, :nq + nk], qkv_p[:, :nq + nk], 1.5 * 2.0 ** -7 * qk_room + 2 * qk_acc),   # a flip before the rotation is rotated too
                 ("o", o, o_p, 3.01 * ulp(o, o_p) + 2e-3 * spread),
                 ("act", act, act_p, None))      # downstream of the differences above: compared in the mean only
        for name, mine, theirs, room in pairs:
            diff = np.abs(mine - theirs)
            frac = float((diff > 0).mean())
            rel_rms = float(np.sqrt((diff ** 2).mean() / (mine ** 2).mean()))
            stats[f"plain_{name}"] = (round(frac, 4), float(f"{rel_rms:.2e}"))
            if room is not None:
                assert (diff <= room + 1e-9).all(), f"layer {l} {name}: MFMA and plain kernels differ by more than rounding ({(diff / (room + 1e-9)).max():.2f} x)"
            # if every element differed by one unit in the last place of bf16 the relative rms difference would be about 3e-3
            assert rel_rms <= 4e-3, f"layer {l} {name}: MFMA and plain kernels differ by {rel_rms:.2e} relative rms"
        dh_ = h_out - d_p.cpu().numpy().astype(np.float64)
        rel = float(np.sqrt((dh_ ** 2).mean() / ((h_out - h_in) ** 2).mean()))
        stats["plain_h_out"] = float(f"{rel:.2e}")
        assert rel <= 4e-3, f"layer {l}: the layer's update differs between MFMA and plain kernels by {rel:.2e} relative rms"
        say(f"[layer] config 3 layer {l}: worst error / bound per stage {stats}; |h| rms {np.sqrt((h_out ** 2).mean()):.3f}; "
            f"{time.perf_counter() - t0:.0f} s")
    model.close()
